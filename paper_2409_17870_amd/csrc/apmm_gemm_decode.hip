// Small-M (decode) kernel, design B: the packed weights are streamed once from HBM and every
// plane pair is multiplied by XOR + popcount on the vector ALU (paper Sec. 3.2 with the XOR form
// of the 1-bit product):
//   D_ij = K - 2 * popcount(a^(j) xor w^(i)),   C = sum_ij 2^(i+j) D_ij
//        = K (2^p - 1)(2^q - 1) - 2 * sum_ij 2^(i+j) popcount(a^(j) xor w^(i)).
// Padded k positions hold equal bits in both operands and drop out of the popcounts.  The
// shift-and-add recovery runs in registers, the reduction over K in registers, lane shuffles
// and LDS; only C reaches global memory (paper Sec. 4.2).
//
// Every kernel of this file takes a group descriptor: several problems of equal p, q can share one launch
// (a workgroup finds its problem from a prefix table of workgroup counts).
//
// Work split.  With M <= 16 tokens the weights (N*K*q/8 bytes) are the only real traffic, a few
// MiB, i.e. a few KiB per CU: the kernel is latency bound, so everything is loaded up front with
// as many waves as possible.
//   workgroup : 16 output channels (half a packed row block), 8 waves
//   wave      : k blocks 4*(w + 8*t) .. +3, t = 0, 1, ...
//   lane l    : weight row l % 16, k block l / 16 of the wave's four; it loads the row's q slots
//               of that block (q x 16 bytes, 256 contiguous bytes per 16 lanes) straight into registers
// The activations (M rows, all K; in passes of a multiple of 32 k blocks when all K does not fit) are copied
// once per workgroup from their packed tiles into LDS with every plane in the common form of the XOR/popcount
// kernels (16 elements per word at the even bit positions, apmm_layout.h); a weight plane is brought to the
// same form after loading, so that any activation plane can be XOR-ed with any weight plane.
#include <hip/hip_ext.h>

#include <algorithm>

#include "apmm_mfma_common.h"

namespace apmm {
namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRowsPerWg = 16;
constexpr int kMaxLdsBytes = 128 * 1024;
constexpr int kMfmaMinTokens = 1;  // the matrix-unit kernel serves every token count its code widths allow

// Words 4*hh .. 4*hh+3 of plane i of an n-bit operand in the common form come from one 16-byte vector of the
// slots of a row and k block (`slots` points at the uint4 of slot 0; consecutive slots are kPlaneWords / 4
// apart): plane_half_src gives its address, plane_half_from turns the loaded vector into the words.
__device__ __forceinline__ const uint4 *plane_half_src(const uint4 *slots, int n, int i, int hh)
{
    constexpr int kSlotVec = kPlaneWords / 4;
    return slots + (i < 2 * pair_groups(n) ? (i / 2 * 2 + hh) : (n - 1)) * kSlotVec;
}

__device__ __forceinline__ uint4 plane_half_from(const uint4 raw, int n, int i, int hh)
{
    if (i < 2 * pair_groups(n)) {
        const uint4 s = raw;  // S[4 hh .. 4 hh + 3] of pair group i / 2
        const int b = i & 1;
        return make_uint4((s.x >> b) & 0x55555555u, (s.y >> b) & 0x55555555u, (s.z >> b) & 0x55555555u,
                          (s.w >> b) & 0x55555555u);
    }
    const uint4 l = raw;
    // word w = 4 hh + x: k step 2 hh + x / 2, words L[2 (x % 2)], L[2 (x % 2) + 1]
    const int k0 = 2 * hh, k1 = 2 * hh + 1;
    return make_uint4(((l.x >> k0) & 0x11111111u) | (((l.y >> k0) & 0x11111111u) << 2),
                      ((l.z >> k0) & 0x11111111u) | (((l.w >> k0) & 0x11111111u) << 2),
                      ((l.x >> k1) & 0x11111111u) | (((l.y >> k1) & 0x11111111u) << 2),
                      ((l.z >> k1) & 0x11111111u) | (((l.w >> k1) & 0x11111111u) << 2));
}

// The same from slots already in registers (weights of a Q-bit operand).
template <int Q>
__device__ __forceinline__ uint4 plane_half_words_reg(const uint4 (&slot)[Q], int i, int hh)
{
    if (i < 2 * pair_groups(Q)) {
        const uint4 s = slot[i / 2 * 2 + hh];
        const int b = i & 1;
        return make_uint4((s.x >> b) & 0x55555555u, (s.y >> b) & 0x55555555u, (s.z >> b) & 0x55555555u,
                          (s.w >> b) & 0x55555555u);
    }
    const uint4 l = slot[Q - 1];
    const int k0 = 2 * hh, k1 = 2 * hh + 1;
    return make_uint4(((l.x >> k0) & 0x11111111u) | (((l.y >> k0) & 0x11111111u) << 2),
                      ((l.z >> k0) & 0x11111111u) | (((l.w >> k0) & 0x11111111u) << 2),
                      ((l.x >> k1) & 0x11111111u) | (((l.y >> k1) & 0x11111111u) << 2),
                      ((l.z >> k1) & 0x11111111u) | (((l.w >> k1) & 0x11111111u) << 2));
}

// The 128 codes of k block kb of activation row m as bytes: d[8 ks + 2 t + jh] holds the codes of elements
// 32 ks + 8 t + 4 jh + (0..3) of the block, masked to `bits` bits; elements past K are the all-ones padding code,
// rows past M are zero.  All loads of a block are issued together (one round trip to memory per block).
__device__ __forceinline__ void load_code_block(const uint8_t *__restrict__ codes, int64_t M, int64_t K, int bits,
                                                int64_t m, int64_t kb, uint32_t (&d)[32])
{
    if (m >= M) {
#pragma unroll
        for (int i = 0; i < 32; ++i) d[i] = 0u;
        return;
    }
    const int64_t k0 = kb * kKBlock;
    const uint8_t *src = codes + m * K + k0;
    if (k0 + kKBlock <= K && ((reinterpret_cast<uintptr_t>(src)) & 15) == 0) {
        uint4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = reinterpret_cast<const uint4 *>(src)[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            d[4 * i] = v[i].x; d[4 * i + 1] = v[i].y; d[4 * i + 2] = v[i].z; d[4 * i + 3] = v[i].w;
        }
    } else {  // ragged end of a row, or a row that does not start at a multiple of 16 bytes: byte by byte
#pragma unroll
        for (int i = 0; i < 32; ++i) d[i] = 0xffffffffu;
        const int64_t left = K - k0;
        const int count = left >= kKBlock ? kKBlock : (left > 0 ? (int)left : 0);
#pragma unroll 1
        for (int e = 0; e < count; ++e) {
            const uint32_t flip = (uint32_t)(src[e] ^ 0xffu) << (8 * (e & 3));
#pragma unroll
            for (int i = 0; i < 32; ++i)
                if (i == (e >> 2)) d[i] ^= flip;
        }
    }
    const uint32_t code_mask = 0x01010101u * ((1u << bits) - 1u);
#pragma unroll
    for (int i = 0; i < 32; ++i) d[i] &= code_mask;
}

// CODES: the activations come as unpacked codes (GemmArgs::a_codes) instead of packed tiles
template <int MT, int Q, bool CODES>
__global__ __launch_bounds__(kThreads) void gemm_decode_kernel(GroupArgs ga)
{
    // Which problem of the launch this workgroup works on (uniform over the workgroup).  Problem 0 is read from
    // fixed kernel-argument offsets, so that a launch of one problem needs a single round of scalar loads before
    // the first weight address is known (every dependent round costs a few hundred ns in a kernel of a few us).
    GemmArgs g = ga.g[0];
    int64_t chunk_kb = ga.chunk_kb[0];
    int block = (int)blockIdx.x;
    if (ga.count > 1) {
        int idx = 0;
        for (int i = 0; i + 1 < ga.count; ++i)
            if ((int)blockIdx.x >= ga.wg_end[i]) idx = i + 1;
        if (idx > 0) {
            g = ga.g[idx];
            chunk_kb = ga.chunk_kb[idx];
            block -= ga.wg_end[idx - 1];
        }
    }
    extern __shared__ __align__(16) uint8_t lds_raw[];
    uint4 *a_lds = reinterpret_cast<uint4 *>(lds_raw);  // [kb][m < MT][j < p][hh < 2] plane words, common form
    const int p = g.p;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n0 = (int64_t)block * kRowsPerWg;

    const int row = lane & 15, sub = lane >> 4;
    int64_t n = n0 + row;
    const int64_t n_ld = n < round_up(g.N, kRowBlock) ? n : round_up(g.N, kRowBlock) - 1;
    constexpr int kSlotVec = kPlaneWords / 4;

    // Order of the requests.  Loads return in order, so whatever is requested before the weights can be used
    // while the weights are still on their way, and whatever is requested after them cannot.  First therefore
    // this thread's first chunk of activations (packed input; usually its only one), which goes to LDS and
    // through a barrier before the k loop; then the weights of the first k block, whose latency is the
    // longest thing in this kernel; then what only the final store needs.
    const uint32_t chunks_per_kb = (uint32_t)(MT * p * 2);
    const uint32_t chunks_pass0 = (uint32_t)(chunk_kb < g.nkb ? chunk_kb : g.nkb) * chunks_per_kb;
    // chunk c of a pass that starts at k block kb0: (k block, row m, plane j, half hh)
    auto chunk_src = [&](uint32_t c, int64_t kb0, uint32_t &j, uint32_t &hh) {
        const uint32_t ckb = c / chunks_per_kb;
        const uint32_t rem = c - ckb * chunks_per_kb, plane = rem >> 1, m = plane / p;
        j = plane - m * p;
        hh = rem & 1;
        const uint4 *slots = reinterpret_cast<const uint4 *>(g.a + tile_row_word(m, kb0 + ckb, g.nkb, p, 0));
        return plane_half_src(slots, p, j, hh);
    };
    uint4 a_first = make_uint4(0, 0, 0, 0);
    uint32_t a_first_j = 0, a_first_hh = 0;
    if constexpr (!CODES) {
        if ((uint32_t)tid < chunks_pass0) a_first = *chunk_src(tid, 0, a_first_j, a_first_hh);
    }

    // (Everything from here to the LDS writes is loaded without a condition, from clamped addresses where the
    // thread has nothing to load: the wait for the activations may leave exactly these loads outstanding only
    // if every thread issues all of them.)
    int64_t kb = 4 * (int64_t)wave + sub;
    uint4 wnext[Q];
    {
        const int64_t kb_ld = kb < g.nkb ? kb : g.nkb - 1;
        const uint4 *wsrc = reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld, kb_ld, g.nkb, Q, 0));
#pragma unroll
        for (int s = 0; s < Q; ++s) wnext[s] = wsrc[s * kSlotVec];
    }

    // What the final store needs is requested now as well (a dependent round trip to memory at the end of a
    // kernel this short would be a quarter of its duration) and kept as loaded: nothing may use the values
    // before the end, or the wave would wait for them here.  A missing scale vector reads a weight word instead.
    const int out_m = tid / kRowsPerWg;
    const int64_t out_n = n0 + tid % kRowsPerWg;
    const bool out_thread = tid < MT * kRowsPerWg && out_m < g.M && out_n < g.N;
    const uint16_t *dummy = reinterpret_cast<const uint16_t *>(g.w);
    uint32_t out_sa_bits = *(g.a_scale ? g.a_scale + (out_m < g.M ? out_m : g.M - 1) : dummy);
    uint32_t out_sw_bits = *(g.w_scale ? g.w_scale + (out_n < g.N ? out_n : g.N - 1) : dummy);

    uint32_t acc[MT];  // sum_ij 2^(i+j) popcount, modulo 2^32
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0;

    // The activations of chunk_kb k blocks at a time sit in LDS (all of K when it fits, which is the usual
    // case): chunk (kb, m, j, hh) = four words of plane j of row m in k block kb.  A pass boundary is a multiple
    // of 32 k blocks, i.e. of the stride of the lanes' k blocks.
    for (int64_t kb0 = 0; kb0 < g.nkb; kb0 += chunk_kb) {
        const int64_t kb_end = kb0 + chunk_kb < g.nkb ? kb0 + chunk_kb : g.nkb;
        if (kb0) __syncthreads();  // every wave is done with the previous pass
        if constexpr (CODES) {
            // straight from the codes: a thread takes the 128 codes of (row m, k block) and writes every plane j in
            // the common form: word w = 2 ks + tp holds elements (ks, t = 2 tp + tt, jh, c) at bit 8c + 4jh + 2tt
            // (32-bit index arithmetic: a pass holds at most 8192 sixteen-byte chunks)
            const uint32_t pass_kb = (uint32_t)(kb_end - kb0), total_blocks = pass_kb * MT;
            for (uint32_t c = tid; c < total_blocks; c += kThreads) {  // consecutive lanes: consecutive 128 bytes of a row
                const uint32_t m = c / pass_kb, ckb = c - m * pass_kb;
                uint32_t d[32];
                load_code_block(g.a_codes, g.M, g.K, p, m, kb0 + ckb, d);
                for (int j = 0; j < p; ++j) {
                    uint32_t word[8];
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        word[w] = 0;
#pragma unroll
                        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                            for (int jh = 0; jh < 2; ++jh)
                                word[w] |= ((d[8 * (w >> 1) + 2 * (2 * (w & 1) + tt) + jh] >> j) & 0x01010101u) << (4 * jh + 2 * tt);
                    }
                    uint4 *dst = a_lds + ckb * chunks_per_kb + (m * p + j) * 2;
                    dst[0] = make_uint4(word[0], word[1], word[2], word[3]);
                    dst[1] = make_uint4(word[4], word[5], word[6], word[7]);
                }
            }
        } else {
            const uint32_t total_chunks = (uint32_t)(kb_end - kb0) * chunks_per_kb;
            uint32_t c = tid;
            if (kb0 == 0) {  // the chunk requested at the top
                if (c < total_chunks) a_lds[c] = plane_half_from(a_first, p, a_first_j, a_first_hh);
                c += kThreads;
            }
            for (; c < total_chunks; c += kThreads) {
                uint32_t j, hh;
                const uint4 raw = *chunk_src(c, kb0, j, hh);
                a_lds[c] = plane_half_from(raw, p, j, hh);
            }
        }
        __syncthreads();

        for (; kb < kb_end; kb += 4 * kWaves) {
            uint4 wraw[Q];
#pragma unroll
            for (int s = 0; s < Q; ++s) wraw[s] = wnext[s];
            if (kb + 4 * kWaves < g.nkb) {  // next block of this lane
                const uint4 *wsrc =
                    reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld, kb + 4 * kWaves, g.nkb, Q, 0));
#pragma unroll
                for (int s = 0; s < Q; ++s) wnext[s] = wsrc[s * kSlotVec];
            }
            uint4 w[Q][2];
#pragma unroll
            for (int i = 0; i < Q; ++i)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) w[i][hh] = plane_half_words_reg<Q>(wraw, i, hh);
            const uint4 *arow = a_lds + (kb - kb0) * chunks_per_kb;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                for (int j = 0; j < p; ++j) {
                    const uint4 a0 = arow[(m * p + j) * 2], a1 = arow[(m * p + j) * 2 + 1];
#pragma unroll
                    for (int i = 0; i < Q; ++i) {
                        const uint32_t pc = __popc(a0.x ^ w[i][0].x) + __popc(a0.y ^ w[i][0].y) +
                                            __popc(a0.z ^ w[i][0].z) + __popc(a0.w ^ w[i][0].w) +
                                            __popc(a1.x ^ w[i][1].x) + __popc(a1.y ^ w[i][1].y) +
                                            __popc(a1.z ^ w[i][1].z) + __popc(a1.w ^ w[i][1].w);
                        acc[m] += pc << (i + j);
                    }
                }
            }
        }
    }

    // reduce over the four k blocks held by the lane groups, then over the waves through LDS
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        acc[m] += __shfl_xor(acc[m], 16);
        acc[m] += __shfl_xor(acc[m], 32);
    }
    __syncthreads();  // every wave is done reading the activations
    uint32_t *part = reinterpret_cast<uint32_t *>(lds_raw);  // [wave][m][row]
    if (lane < 16) {
#pragma unroll
        for (int m = 0; m < MT; ++m) part[(wave * MT + m) * kRowsPerWg + lane] = acc[m];
    }
    __syncthreads();
    if (out_thread) {
        uint32_t s = 0;
#pragma unroll
        for (int w8 = 0; w8 < kWaves; ++w8) s += part[(w8 * MT + out_m) * kRowsPerWg + tid % kRowsPerWg];
        const uint32_t full = (uint32_t)g.K * (uint32_t)((1 << p) - 1) * (uint32_t)((1 << Q) - 1);
        out_sa_bits = g.a_scale ? use_here(out_sa_bits) : 0x3c00u;  // 1.0
        out_sw_bits = g.w_scale ? use_here(out_sw_bits) : 0x3c00u;
        store_output(g, out_m, out_n, (int32_t)(full - 2u * s), half_bits_to_float((uint16_t)out_sa_bits),
                     half_bits_to_float((uint16_t)out_sw_bits));
    }
}

// k blocks of activations per pass: all of K when that fits the LDS budget, else the largest multiple of 32
// (the k-block stride of the lanes) that does; `per_kb` = LDS bytes of one k block, `extra` = bytes beside them.
int64_t pass_k_blocks(int64_t nkb, size_t per_kb, size_t extra)
{
    const int64_t fit = (int64_t)((kMaxLdsBytes - extra) / per_kb);
    if (nkb <= fit) return nkb;
    return fit / (4 * kWaves) * (4 * kWaves);  // 0: not even one stride fits
}

int64_t decode_pass_kb(const GemmArgs &g, int mt) { return pass_k_blocks(g.nkb, (size_t)mt * g.p * 32, 0); }

size_t decode_lds_bytes(const GemmArgs &g, int mt)
{
    const size_t a_bytes = (size_t)decode_pass_kb(g, mt) * mt * g.p * 32;
    const size_t part_bytes = (size_t)kWaves * mt * kRowsPerWg * 4;
    return a_bytes > part_bytes ? a_bytes : part_bytes;
}

int decode_mt(int64_t M) { return M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : 16; }

// Builds the launch descriptor of `count` problems (16 output channels per workgroup each).
template <class PassKb>
bool make_group(const GemmArgs *gs, int count, int rows_per_wg, PassKb pass_kb, GroupArgs &ga)
{
    if (count < 1 || count > kMaxGroup) return false;
    int64_t end = 0;
    ga.count = count;
    for (int i = 0; i < kMaxGroup; ++i) {
        const GemmArgs &g = gs[i < count ? i : count - 1];
        if (i < count) end += (g.N + rows_per_wg - 1) / rows_per_wg;
        if (end > 0x7fffffffLL) return false;
        ga.wg_end[i] = (int)end;
        ga.g[i] = g;
        ga.chunk_kb[i] = (int)pass_kb(g);
        if (ga.chunk_kb[i] < 1) return false;
    }
    return true;
}

template <class Kernel>
hipError_t launch_group(Kernel kernel, bool &attr_set, const GroupArgs &ga, size_t lds, hipStream_t stream)
{
    if (!attr_set) {  // idempotent; a race here is harmless
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const KernelTiming timing = take_kernel_timing();
    if (timing.start || timing.stop)
        hipExtLaunchKernelGGL(kernel, dim3((unsigned)ga.wg_end[ga.count - 1]), dim3(kThreads), lds, stream,
                              timing.start, timing.stop, 0, ga);
    else
        hipLaunchKernelGGL(kernel, dim3((unsigned)ga.wg_end[ga.count - 1]), dim3(kThreads), lds, stream, ga);
    return hipGetLastError();
}

template <int MT, int Q>
hipError_t launch_mt_q(const GroupArgs &ga, hipStream_t stream)
{
    size_t lds = 0;
    for (int i = 0; i < ga.count; ++i) lds = lds > decode_lds_bytes(ga.g[i], MT) ? lds : decode_lds_bytes(ga.g[i], MT);
    static bool attr_set[2] = {false, false};
    note_kernel("gemm_decode_kernel<%d,%d,%s>", MT, Q, ga.g[0].a_codes ? "codes" : "packed");
    if (ga.g[0].a_codes) return launch_group(gemm_decode_kernel<MT, Q, true>, attr_set[1], ga, lds, stream);
    return launch_group(gemm_decode_kernel<MT, Q, false>, attr_set[0], ga, lds, stream);
}

template <int MT>
hipError_t launch_mt(const GroupArgs &ga, hipStream_t stream)
{
    switch (ga.g[0].q) {
    case 1: return launch_mt_q<MT, 1>(ga, stream);
    case 2: return launch_mt_q<MT, 2>(ga, stream);
    case 3: return launch_mt_q<MT, 3>(ga, stream);
    case 4: return launch_mt_q<MT, 4>(ga, stream);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Small-M kernel on the matrix unit (M <= 64, p, q <= 2).  With more than a couple of tokens the
// XOR/popcount form needs 2 p q M lane-operations per weight word and becomes VALU bound; the E2M1 MFMA
// needs one expansion of the weight words (1.25 - 1.5 operations per 8 codes) whatever M is.
// Same split of the work as the XOR/popcount kernel (8 waves over K, lane = weight row l % 16 and k block
// l / 16 of four), same algebra as the large-M MFMA kernel:
//   v_mfma_scale_f32_16x16x128_f8f6f4: A = 16 weight rows x 128 k, B = 128 k x 16 tokens, codes as E2M1;
//   MFMA ks of an iteration multiplies k step ks of the four k blocks held by the four lane groups;
//   a workgroup owns RT tiles of 16 output channels and all TT tiles of 16 tokens: a weight fragment is
//   expanded once and multiplied with TT token fragments, a token fragment with RT weight fragments;
//   C = acc - 2 cw PA[m] - 2 ca PW[n] + K ca cw with the packed row sums (the operand scales make acc = 4 S).
// No staging through LDS and no barrier before the k loop: the waves split K, so every (token, k block)
// fragment of the activations is consumed by exactly one lane group of one wave, which loads it straight
// from global memory (L2) like its weights: lane (r16, kq) takes the P slots of token 16 tt + r16 in its
// k block, 256 contiguous bytes per 16 lanes.  Everything a wave needs is requested in its first
// instructions; the only barrier is the one of the cross-wave reduction at the end.
// With activation codes as input (CODES = 1, or 2 for rows that allow no aligned 16-byte loads) a wave loads
// the codes of its group of four k blocks together, turns every 16 codes into the packed word they form and
// passes the words to the lanes that need them through LDS of its own (see load_chunks); the tokens' code
// sums PA[m], which the packed operand would have carried, come from one more MFMA per k step against a
// weight fragment of all-one codes.  NJ = 1 is the variant for at most two tokens: one chunk per lane, few
// enough registers for three workgroups per CU.
// The first problem's arguments are plain kernel arguments ahead of the group descriptor: this file is built
// with kernel-argument preloading, so the first 14 dwords of the kernel-argument segment are in scalar
// registers when the wave starts and a single-problem launch computes its first addresses without a round
// trip to memory for its arguments (measured: 0.3 us of a 3.4 us launch).
// RT = 2 halves the number of workgroups when there are plenty of output channels.
// Measured against the version that staged the activations of all K through LDS behind a workgroup barrier
// (W2A2, us per launch inside a graph, cold weights; 4096 x 4096 / 11008 x 4096 / 4096 x 11008): packed
// operands, 8 tokens 3.6 -> 3.1 / 5.1 -> 4.4 / 5.8 -> 4.6; from codes, 1 token (then on the XOR/popcount
// kernel) 4.3 -> 3.2 / 7.6 -> 4.7 / 6.1 -> 4.9, 16 tokens 5.7 -> 4.4 / 9.8 -> 7.3 / 10.1 -> 7.1.
// ---------------------------------------------------------------------------------------------
struct DecodeProblem {
    const uint32_t *w;
    const void *a;          // packed activations, or codes (CODES)
    int64_t N, K, M;
    uint16_t *c_f16;
    int32_t *c_i32;
    const uint16_t *w_scale, *a_scale;
};

// problem of this workgroup and its index among the problem's workgroups
__device__ __forceinline__ int pick_problem(DecodeProblem &pr, uint32_t misc, const GroupArgs &ga)
{
    int block = (int)blockIdx.x;
    const int count = (int)((misc >> 12) & 0xffu);
    if (count > 1) {
        int idx = 0;
        for (int i = 0; i + 1 < count; ++i)
            if ((int)blockIdx.x >= ga.wg_end[i]) idx = i + 1;
        if (idx > 0) {
            const GemmArgs &g = ga.g[idx];
            pr.w = g.w;
            pr.a = g.a_codes ? static_cast<const void *>(g.a_codes) : static_cast<const void *>(g.a);
            pr.N = g.N; pr.K = g.K; pr.M = g.M;
            pr.c_f16 = g.c_f16; pr.c_i32 = g.c_i32;
            pr.w_scale = g.w_scale; pr.a_scale = g.a_scale;
            block -= ga.wg_end[idx - 1];
        }
    }
    return block;
}

template <int P, int Q, int TT, int RT, int CODES, int NJ = 8>
__global__ __launch_bounds__(kThreads, (CODES == 1 && TT == 1) ? (NJ == 1 && RT == 1 ? 6 : 4) - (Q > 2 ? 1 : 0) : 2)  // waves per SIMD aimed at (weights of two plane groups hold twice the raw words)
void gemm_decode_mfma_kernel(const uint32_t *w_arg, const void *a_arg, int n_arg, int k_arg,
                             uint32_t misc_arg /* M | problems << 12 | token groups << 24 */, int reserved_arg, uint16_t *cf_arg, int32_t *ci_arg,
                             const uint16_t *ws_arg, const uint16_t *as_arg, GroupArgs ga)
{
    static_assert((P <= 2 || (activation_field_form(P) && NJ == 8)) && Q <= 4,
                  "one plane group per activation, or activations in the field form (ready-made E2M3 operands); "
                  "weights of one or two plane groups");
    constexpr int WS = Q > 2 ? Q : 2;        // weight slots held per channel tile
    constexpr int NG = pair_groups(Q) + (has_single_group(Q) ? 1 : 0);  // plane groups of the weights
    constexpr bool AF = activation_field_form(P);
    constexpr int SA = activation_slots(P);  // slots of an activation row and k block
    static_assert(NJ == 8 || (NJ == 1 && CODES == 1 && TT == 1), "NJ = 1: codes of at most two tokens");
    (void)reserved_arg;
    DecodeProblem pr = {w_arg, a_arg, n_arg, k_arg, (int64_t)(misc_arg & 0xfffu), cf_arg, ci_arg, ws_arg, as_arg};
    int block = pick_problem(pr, misc_arg, ga);
    constexpr int ROWS = kRowsPerWg * RT;
    // Token groups (packed operands, one problem per launch): with more tokens than the TT tiles of a workgroup hold,
    // the grid is repeated per group of 16 TT tokens; a workgroup re-reads its 16 or 32 packed weight rows (from L2,
    // a few KiB) and works on tokens tok0 ... of the same packed operands and outputs.
    int tok0 = 0;
    if constexpr (!CODES) {
        if ((misc_arg >> 24) > 1) {
            const int per_group = (int)((pr.N + ROWS - 1) / ROWS);
            tok0 = (block / per_group) * 16 * TT;
            block %= per_group;
        }
    }
    constexpr int OUTS = (TT * RT * 256 + kThreads - 1) / kThreads;  // outputs per thread
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    constexpr int kSlotVec = kPlaneWords / 4;
    extern __shared__ __align__(16) uint8_t lds_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t n0 = (int64_t)block * ROWS;
    const int64_t nkb = ((pr.K + kKPad - 1) / kKPad) * (kKPad / kKBlock);
    const int64_t rows_a = round_up(pr.M, kRowBlock), rows_b = round_up(pr.N, kRowBlock);

    // this lane's weight rows and tokens, at its k block of the wave's first group of four
    const int groups = (int)(nkb / 4);                       // groups of four k blocks; the waves take them in turn
    const int iters = groups > wave ? (groups - wave + kWaves - 1) / kWaves : 0;
    const uint4 *wsrc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int64_t n = n0 + rt * 16 + r16 < rows_b ? n0 + rt * 16 + r16 : rows_b - 1;
        wsrc[rt] = reinterpret_cast<const uint4 *>(pr.w + tile_row_word(n, 4 * wave + kq, nkb, Q, 0));
    }
    constexpr int kIterVecW = 4 * kWaves * Q * kSlotVec;     // uint4 between this lane's k blocks of consecutive iterations
    constexpr int kIterVecA = 4 * kWaves * SA * kSlotVec;
    const uint4 *asrc[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        asrc[tt] = nullptr;
        if constexpr (!CODES) {
            // tokens past M: the padded rows of the last row block hold zero words (read, never stored)
            const int64_t t = tok0 + tt * 16 + r16, t_ld = t < rows_a ? t : rows_a - 1;
            asrc[tt] = reinterpret_cast<const uint4 *>(static_cast<const uint32_t *>(pr.a) +
                                                       tile_row_word(t_ld, 4 * wave + kq, nkb, SA, 0));
        }
    }

    uint4 wnext[RT][WS], anext[TT][AF ? 6 : 2];
    auto load_packed = [&](int it) __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int s = 0; s < Q; ++s) wnext[rt][s] = wsrc[rt][(int64_t)it * kIterVecW + s * kSlotVec];
        if constexpr (!CODES) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int s = 0; s < SA; ++s) anext[tt][s] = asrc[tt][(int64_t)it * kIterVecA + s * kSlotVec];
        }
    };
    // CODES.  The codes of one token tile and one group of four k blocks are 16 runs of 512 contiguous bytes
    // (one per token).  The wave loads them together, lane l taking chunk l % 32 (16 codes) of token 2 j + l / 32 in
    // its j-th load: every load instruction reads two whole runs.  The 16 codes of a chunk are exactly one packed
    // word of their row and k block (word w = chunk % 8 of k block chunk / 8: apmm_layout.h), so a lane turns
    // each chunk into that word with seven operations and the words change lanes through a piece of LDS that
    // belongs to the wave alone (no workgroup barrier): lane (r16, kq) reads back the eight words of token r16 in
    // k block kq, its MFMA fragment.
    // per wave: [token 16][k block 4][word 8] (single group: two partial words each; field form: 24 words)
    constexpr int kXposeWords = AF ? 1536 : P == 1 ? 1024 : 512;
    uint32_t *xpose = reinterpret_cast<uint32_t *>(lds_raw) + kWaves * RT * TT * 256 + kWaves * TT * 16 + wave * kXposeWords;
    // CODES == 1: K is a multiple of 16 and the matrix starts at a multiple of 16 bytes, so every chunk is one
    // aligned 16-byte load and lies wholly inside the row or wholly in the padding.  The loads are issued without
    // any condition on the lane (lanes with nothing to load read the first chunk of the matrix instead and mask it
    // away at the point of use): a load inside a divergent branch makes the wave wait for it, and for everything
    // requested before it, at the end of the branch.
    // CODES == 2: any K and alignment, byte by byte (correct, slow).
    auto load_chunks = [&](int tt, int it, uint4 (&v)[NJ]) __attribute__((always_inline)) {
        const int64_t k0 = (int64_t)4 * kKBlock * (wave + (int64_t)kWaves * it) + 16 * (lane & 31);
        const int64_t m_tile = pr.M - tt * 16;  // tokens of this tile that exist
        // (the row length as an opaque value: the addresses are then formed where they are used instead of being
        // kept in registers across the k loop, two registers per load and token tile)
        int64_t row_len = pr.K;
        asm volatile("" : "+s"(row_len));
        // CODES == 1: one 32-bit lane offset serves all eight loads; the token pair's row is a uniform base.  Lanes
        // with nothing to load (odd token past M, chunk in the padding) read the first chunk of the pair's first
        // token, which exists whenever the load is issued at all.
        uint32_t lane_off = 0;
        if (k0 + 16 <= row_len) lane_off = (uint32_t)((lane >> 5) * row_len + k0);
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int64_t t = tt * 16 + 2 * jj + (lane >> 5);
            if constexpr (CODES == 1) {
                const uint8_t *pair_row = static_cast<const uint8_t *>(pr.a) + (int64_t)(tt * 16 + 2 * jj) * row_len;  // uniform
                const uint32_t off = t < pr.M ? lane_off : 0u;
                if (2 * jj < m_tile) v[jj] = *reinterpret_cast<const uint4 *>(pair_row + off);  // uniform: token pairs that exist
                else v[jj] = make_uint4(0, 0, 0, 0);
            } else {
                uint32_t d[4] = {0u, 0u, 0u, 0u};  // tokens past M: zero words, as the padded rows of a packed operand
                if (t < pr.M) {
                    const uint8_t *src = static_cast<const uint8_t *>(pr.a) + t * row_len + k0;
                    const int64_t left = row_len - k0;
                    const int count = left >= 16 ? 16 : (left > 0 ? (int)left : 0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) d[i] = 0xffffffffu;  // positions past K hold the all-ones padding code
#pragma unroll 1
                    for (int e = 0; e < count; ++e) {
                        const uint32_t flip = (uint32_t)(src[e] ^ 0xffu) << (8 * (e & 3));
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (i == (e >> 2)) d[i] ^= flip;
                    }
                }
                v[jj] = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
    };
    auto chunks_to_fragment = [&](int tt, int it, const uint4 (&v)[NJ], uint4 (&aq)[AF ? 6 : 2]) __attribute__((always_inline)) {
        constexpr uint32_t code_mask = 0x01010101u * ca;
        // the wave's previous fragment has been read by every lane before anything is overwritten
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int w = lane & 7, slot = ((lane >> 5) * 4 + ((lane & 31) >> 3)) * 8 + w;  // + 64 jj: token 2 jj + l / 32
        const int64_t k0 = (int64_t)4 * kKBlock * (wave + (int64_t)kWaves * it) + 16 * (lane & 31);
        const bool inside = k0 + 16 <= pr.K;
        const int64_t m_tile = pr.M - tt * 16;
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            if (2 * jj >= m_tile) continue;  // uniform; the slots of tokens that do not exist are never stored outputs
            // what the lane loaded counts only for a token that exists and a chunk inside the row; a chunk in the
            // padding of an existing token holds the all-ones code, a token past M zero words
            uint32_t m_and = code_mask, m_or = 0u;
            if constexpr (CODES == 1) {
                const bool valid = tt * 16 + 2 * jj + (lane >> 5) < pr.M;
                m_and = valid && inside ? code_mask : 0u;
                m_or = valid && !inside ? code_mask : 0u;
            }
            // dword i = 2 t2 + jh of the chunk holds the elements (t = 2 tp + t2, jh, c = 0..3) of the word
            const uint32_t d0 = (v[jj].x & m_and) | m_or, d1 = (v[jj].y & m_and) | m_or, d2 = (v[jj].z & m_and) | m_or,
                           d3 = (v[jj].w & m_and) | m_or;
            if constexpr (AF) {
                // Field form: the chunk's 16 codes are the fields 16 tp ... 16 tp + 15 of k step w / 2 (tp = w % 2), i.e. words
                // 6 (w / 2) + 3 tp ... + 2 of the row's 24: byte c of dword i goes to field 8 (i / 2) + 2 c + i % 2, six bits each.
                auto spread12 = [](uint32_t x) __attribute__((always_inline)) {  // byte c -> bits 12 c ... 12 c + 7
                    return (uint64_t)((x & 0xffu) | ((x & 0xff00u) << 4) | ((x & 0xff0000u) << 8)) | ((uint64_t)(x >> 24) << 36);
                };
                const uint64_t lo = spread12(d0) | (spread12(d1) << 6), hi = spread12(d2) | (spread12(d3) << 6);  // 48 bits each
                const int token = 2 * jj + (lane >> 5), kb = (lane & 31) >> 3;
                uint32_t *dst = xpose + (token * 4 + kb) * 24 + 6 * (w >> 1) + 3 * (w & 1);
                dst[0] = (uint32_t)lo;
                dst[1] = (uint32_t)(lo >> 32) | ((uint32_t)hi << 16);
                dst[2] = (uint32_t)(hi >> 16);
            } else if constexpr (P == 2) {
                // S[w]: bit b of element (t2, jh, c) at 8c + 4jh + 2 t2 + b
                xpose[64 * jj + slot] = d0 | (d1 << 4) | (d2 << 2) | (d3 << 6);
            } else {
                // L[2 tp], L[2 tp + 1]: the bit of element (ks, t, jh, c) at 8c + 4jh + ks; this chunk is k step w / 2
                const int ks = w >> 1;
                *reinterpret_cast<uint2 *>(xpose + 2 * (64 * jj + slot)) = make_uint2((d0 | (d1 << 4)) << ks, (d2 | (d3 << 4)) << ks);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int mine = (r16 * 4 + kq) * 8;
        if constexpr (AF) {
#pragma unroll
            for (int i = 0; i < 6; ++i) aq[i] = *reinterpret_cast<const uint4 *>(xpose + 3 * mine + 4 * i);
        } else if constexpr (P == 2) {
            aq[0] = *reinterpret_cast<const uint4 *>(xpose + mine);
            aq[1] = *reinterpret_cast<const uint4 *>(xpose + mine + 4);
        } else {
            uint4 q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) q[i] = *reinterpret_cast<const uint4 *>(xpose + 2 * mine + 4 * i);
            // q[i] = (first, second partial of word 2i, first, second partial of word 2i + 1); words with even w feed
            // L[0], L[1], words with odd w L[2], L[3]
            aq[0] = make_uint4(q[0].x | q[1].x | q[2].x | q[3].x, q[0].y | q[1].y | q[2].y | q[3].y,
                               q[0].z | q[1].z | q[2].z | q[3].z, q[0].w | q[1].w | q[2].w | q[3].w);
        }
    };

    // Order of the requests: weights and activations of the first iteration, then what only the final store
    // needs (kept as loaded: nothing may use those values before the end, or the wave would wait for them here).
    // one token tile: the chunks of the next iteration are requested as soon as those of the current one have been
    // turned into words (their registers are free from then on), ahead of the MFMAs
    uint4 vcur[CODES && TT == 1 ? NJ : 1];
    if (iters > 0) {
        load_packed(0);
        if constexpr (CODES && TT == 1) load_chunks(0, 0, vcur);
    }
    bool out_ok[OUTS];
    int out_m[OUTS];
    int64_t out_n[OUTS];
    uint32_t out_sa_bits[OUTS], out_sw_bits[OUTS], out_pa[OUTS], out_pw[OUTS];
    {
        const int32_t *w_sum = reinterpret_cast<const int32_t *>(pr.w + row_sum_word(rows_b, nkb, Q));
        const int32_t *a_sum = CODES ? nullptr
                                     : reinterpret_cast<const int32_t *>(static_cast<const uint32_t *>(pr.a) +
                                                                         row_sum_word(rows_a, nkb, SA));
        const uint16_t *dummy = reinterpret_cast<const uint16_t *>(pr.w);
#pragma unroll
        for (int o = 0; o < OUTS; ++o) {
            // output o of this thread is element (tile t = e / 256, register v, lane l) of the accumulators,
            // t = rt * TT + tt; 16x16 accumulator layout: lane l, register v holds row 4*(l/16) + v (weight row),
            // column l%16 (token)
            const int e = tid + o * kThreads, t = e >> 8, v = (e >> 6) & 3, l = e & 63;
            out_m[o] = tok0 + (t % TT) * 16 + (l & 15);
            out_n[o] = n0 + (t / TT) * 16 + 4 * (l >> 4) + v;
            out_ok[o] = t < TT * RT && out_m[o] < pr.M && out_n[o] < pr.N;
            const int64_t m_c = out_m[o] < rows_a ? out_m[o] : rows_a - 1, n_c = out_n[o] < rows_b ? out_n[o] : rows_b - 1;
            out_pa[o] = 0;
            if constexpr (!CODES) out_pa[o] = (uint32_t)a_sum[m_c];
            out_pw[o] = (uint32_t)w_sum[n_c];
            out_sa_bits[o] = *(pr.a_scale ? pr.a_scale + (m_c < pr.M ? m_c : pr.M - 1) : dummy);
            out_sw_bits[o] = *(pr.w_scale ? pr.w_scale + (n_c < pr.N ? n_c : pr.N - 1) : dummy);
        }
    }

    mfma::v4f acc[RT][TT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma::v4f{0.f, 0.f, 0.f, 0.f};
    // CODES: the tokens' code sums PA[m] come from the matrix unit as well: one more MFMA per k step against a
    // weight fragment of all-one codes gives 4 PA[token] in every row
    mfma::v4f acc_pa[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) acc_pa[tt] = mfma::v4f{0.f, 0.f, 0.f, 0.f};

    for (int it = 0; it < iters; ++it) {
        uint4 wq[RT][WS], aq[TT][AF ? 6 : 2];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int s = 0; s < Q; ++s) wq[rt][s] = wnext[rt][s];
        if constexpr (!CODES) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int s = 0; s < SA; ++s) aq[tt][s] = anext[tt][s];
        }
        if constexpr (CODES && TT == 1) {
            if (it + 1 < iters) load_packed(it + 1);
            chunks_to_fragment(0, it, vcur, aq[0]);
            if (it + 1 < iters) load_chunks(0, it + 1, vcur);
        } else {
            if (it + 1 < iters) load_packed(it + 1);
            if constexpr (CODES) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    uint4 v[NJ];
                    load_chunks(tt, it, v);
                    chunks_to_fragment(tt, it, v, aq[tt]);
                    __builtin_amdgcn_sched_barrier(0);  // one tile's chunks in registers at a time
                }
            }
        }
        mfma::static_for<4>([&](auto ks_c) __attribute__((always_inline)) {
            constexpr int ks = decltype(ks_c)::value;
            mfma::v8i b8[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) b8[tt] = mfma::v8i{0, 0, 0, 0, 0, 0, 0, 0};
            mfma::static_for<4>([&](auto d_c) __attribute__((always_inline)) {
                constexpr int d = decltype(d_c)::value;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    if constexpr (AF) {
                    } else if constexpr (P == 1) {
                        b8[tt][d] = (int)mfma::fp4_single_dword<ks, d>(aq[tt][0]);
                    } else {
                        b8[tt][d] = (int)mfma::fp4_pair_dword<ks, d>(aq[tt][0], aq[tt][1]);
                    }
                }
            });
            if constexpr (AF) {
                // field form: words 6 ks .. 6 ks + 5 of the lane's 24 are the E2M3 operand of this k step as they stand
                mfma::static_for<6>([&](auto w_c) __attribute__((always_inline)) {
                    constexpr int w = 6 * ks + decltype(w_c)::value;
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) b8[tt][decltype(w_c)::value] = (int)mfma::vec_word<w & 3>(aq[tt][w >> 2]);
                });
            }
            // One MFMA per plane group of the weights (pair groups at code bits 2 g, a single group at bit Q - 1), all into
            // the same accumulator: the group's bit position goes into the weights' power-of-two operand scale.
            // E8M0 exponents: 2^2 per operand turns (ua/2)(uw/2) into 4 ua uw; field form: (ua/8)(uw/2) 2^6.
            // Operand formats: 4 = E2M1, 2 = E2M3.
            mfma::static_for<NG>([&](auto g_c) __attribute__((always_inline)) {
                constexpr int grp = decltype(g_c)::value;
                constexpr bool SINGLE = grp >= pair_groups(Q);
                constexpr int slot = SINGLE ? Q - 1 : 2 * grp;
                mfma::v8i a8[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) a8[rt] = mfma::v8i{0, 0, 0, 0, 0, 0, 0, 0};
                mfma::static_for<4>([&](auto d_c) __attribute__((always_inline)) {
                    constexpr int d = decltype(d_c)::value;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        if constexpr (SINGLE) a8[rt][d] = (int)mfma::fp4_single_dword<ks, d>(wq[rt][slot]);
                        else a8[rt][d] = (int)mfma::fp4_pair_dword<ks, d>(wq[rt][slot], wq[rt][slot + 1]);
                    }
                });
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        acc[rt][tt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                            a8[rt], b8[tt], acc[rt][tt], 4, AF ? 2 : 4, 0,
                            (AF ? 130 : 129) + slot + (SINGLE ? mfma::fp4_single_exponent(ks) : 0), 0,
                            AF ? 130 : 129 + (P == 1 ? mfma::fp4_single_exponent(ks) : 0));
            });
            if constexpr (CODES) {
                const mfma::v8i ones = {0x11111111, 0x11111111, 0x11111111, 0x11111111, 0, 0, 0, 0};  // E2M1 0.5 = the code 1
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    acc_pa[tt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        ones, b8[tt], acc_pa[tt], 4, AF ? 2 : 4, 0, AF ? 130 : 129, 0,
                        AF ? 130 : 129 + (P == 1 ? mfma::fp4_single_exponent(ks) : 0));
            }
        });
    }

    // reduce over the waves through LDS: part[wave][tile t][v][lane], and (CODES) the code sums pa[wave][token]
    float *part = reinterpret_cast<float *>(lds_raw);
    uint32_t *pa_lds = reinterpret_cast<uint32_t *>(lds_raw) + kWaves * RT * TT * 256;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[((wave * RT * TT + rt * TT + tt) * 4 + v) * 64 + lane] = acc[rt][tt][v];
    if constexpr (CODES) {
        // register 0 of lanes 0 .. 15 is row 0, token = lane: 4 PA[token], an integer below 2^24
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
            if (lane < 16) pa_lds[wave * TT * 16 + tt * 16 + lane] = (uint32_t)(int32_t)acc_pa[tt][0] >> 2;
    }
    __syncthreads();
#pragma unroll
    for (int o = 0; o < OUTS; ++o) {
        if (!out_ok[o]) continue;
        const int e = tid + o * kThreads;  // = (t * 4 + v) * 64 + l
        float s = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < kWaves; ++w8) s += part[w8 * RT * TT * 256 + e];
        uint32_t pa = out_pa[o];
        if constexpr (CODES) {
            pa = 0;
#pragma unroll
            for (int w8 = 0; w8 < kWaves; ++w8) pa += pa_lds[w8 * TT * 16 + out_m[o]];
        } else {
            pa = use_here(pa);
        }
        // C = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw
        const uint32_t terms = (uint32_t)pr.K * ca * cw - 2u * cw * pa - 2u * ca * use_here(out_pw[o]);
        const uint32_t sa_bits = pr.a_scale ? use_here(out_sa_bits[o]) : 0x3c00u;  // 1.0
        const uint32_t sw_bits = pr.w_scale ? use_here(out_sw_bits[o]) : 0x3c00u;
        const int32_t c = (int32_t)((uint32_t)(int32_t)s + terms);
        const int64_t at = (int64_t)out_m[o] * pr.N + out_n[o];
        if (pr.c_i32) pr.c_i32[at] = c;
        if (pr.c_f16)
            pr.c_f16[at] = float_to_half_bits((float)c * half_bits_to_float((uint16_t)sa_bits) *
                                              half_bits_to_float((uint16_t)sw_bits));
    }
}

// token tiles of 16 per workgroup, and groups of that many tokens per launch (packed operands only)
int decode_token_tiles(const GemmArgs &g) { return g.M <= 16 ? 1 : (g.M <= 32 || activation_field_form(g.p)) ? 2 : 4; }
int decode_token_groups(const GemmArgs &g) { return (int)((g.M + 16 * decode_token_tiles(g) - 1) / (16 * decode_token_tiles(g))); }
// (measured, W2A2 / W2A4 against the K-split kernel at 4096 x 4096: two groups of 64 tokens 7.5 - 8.0 against 7.8 - 8.5 us,
// three and four groups 11.3 - 14.7 against 7.9 - 8.1 us; two groups of 32 tokens with 4-bit activations 6.4 - 6.6 against
// 9.4 - 10.2 us: only the last is offered)
constexpr int kMaxTokenGroups = 2;

size_t decode_mfma_lds_bytes(const GemmArgs &g, int rt)
{
    const int tt = decode_token_tiles(g);
    // accumulator partials + code sums + (codes) the waves' exchange areas
    return (size_t)kWaves * rt * tt * 256 * 4 + (size_t)kWaves * tt * 16 * 4 + (g.a_codes ? (size_t)kWaves * (activation_field_form(g.p) ? 6144 : g.p == 1 ? 4096 : 2048) : 0);
}

// 1- and 2-bit codes, up to 64 tokens; packed 3- and 4-bit activations (field form) with 1- and 2-bit weights, 32
// tokens per workgroup (two token tiles: their 24 words per row and k block leave no registers for four) and up to
// two such token groups per launch
bool decode_mfma_supported(const GemmArgs &g)
{
    const bool widths = g.q <= 4 && (g.p <= 2 || activation_field_form(g.p));
    const int64_t per_wg = activation_field_form(g.p) ? 32 : 64;
    return g.M >= kMfmaMinTokens && g.M <= (activation_field_form(g.p) && !g.a_codes ? kMaxTokenGroups * per_wg : per_wg) && widths && g.K <= 0x7fffffffLL && g.N <= 0x7fffffffLL &&
           4 * g.nkb * kKBlock * ((1 << g.p) - 1) * ((1 << g.q) - 1) < (1 << 24);
}

template <class Kernel>
hipError_t launch_group_scalars(Kernel kernel, bool &attr_set, const GroupArgs &ga, size_t lds, hipStream_t stream)
{
    if (!attr_set) {  // idempotent; a race here is harmless
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const GemmArgs &g = ga.g[0];
    const void *a = g.a_codes ? static_cast<const void *>(g.a_codes) : static_cast<const void *>(g.a);
    const int groups = ga.count == 1 && !g.a_codes ? decode_token_groups(g) : 1;
    const uint32_t misc = (uint32_t)g.M | ((uint32_t)ga.count << 12) | ((uint32_t)groups << 24);
    if ((int64_t)ga.wg_end[ga.count - 1] * groups > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(ga.wg_end[ga.count - 1] * groups)), block(kThreads);
    const KernelTiming timing = take_kernel_timing();
    if (timing.start || timing.stop)
        hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, timing.start, timing.stop, 0, g.w, a, (int)g.N, (int)g.K,
                              misc, 0, g.c_f16, g.c_i32, g.w_scale, g.a_scale, ga);
    else
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, g.w, a, (int)g.N, (int)g.K, misc, 0, g.c_f16, g.c_i32,
                           g.w_scale, g.a_scale, ga);
    return hipGetLastError();
}

template <int P, int Q, int TT, int RT>
hipError_t launch_decode_mfma_v(const GroupArgs &ga, hipStream_t stream)
{
    size_t lds = 0;
    for (int i = 0; i < ga.count; ++i)
        lds = lds > decode_mfma_lds_bytes(ga.g[i], RT) ? lds : decode_mfma_lds_bytes(ga.g[i], RT);
    static bool attr_set[4] = {false, false, false, false};
    note_kernel("gemm_decode_mfma_kernel<%d,%d,%d,%d,%s>", P, Q, TT, RT, ga.g[0].a_codes ? "codes" : "packed");
    if constexpr (activation_field_form(P)) {  // from codes: single channel tiles only
        if (ga.g[0].a_codes) {
            if constexpr (RT == 1) {
                bool vec_ok = true;
                for (int i = 0; i < ga.count; ++i)
                    vec_ok = vec_ok && (ga.g[i].K & 15) == 0 && (reinterpret_cast<uintptr_t>(ga.g[i].a_codes) & 15) == 0;
                if (vec_ok) return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 1>, attr_set[1], ga, lds, stream);
                return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 2>, attr_set[2], ga, lds, stream);
            } else {
                return hipErrorInvalidValue;
            }
        }
        return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 0>, attr_set[0], ga, lds, stream);
    } else
    if (ga.g[0].a_codes) {
        // (four token tiles from codes with two row tiles would not fit the registers: the launcher never asks for it)
        if constexpr (TT == 4 && RT == 2) {
            return hipErrorInvalidValue;
        } else {
            // one aligned 16-byte load per chunk when every problem's rows allow it, else the byte-wise variant
            bool vec_ok = true;
            for (int i = 0; i < ga.count; ++i)
                vec_ok = vec_ok && (ga.g[i].K & 15) == 0 && (reinterpret_cast<uintptr_t>(ga.g[i].a_codes) & 15) == 0;
            if constexpr (TT == 1) {
                // at most two tokens everywhere: the variant that loads one chunk per lane (fewer registers, three
                // workgroups per CU)
                bool two = vec_ok;
                for (int i = 0; i < ga.count; ++i) two = two && ga.g[i].M <= 2;
                if (two) return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 1, 1>, attr_set[3], ga, lds, stream);
            }
            if (vec_ok) return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 1>, attr_set[1], ga, lds, stream);
            return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 2>, attr_set[2], ga, lds, stream);
        }
    }
    return launch_group_scalars(gemm_decode_mfma_kernel<P, Q, TT, RT, 0>, attr_set[0], ga, lds, stream);
}

template <int P, int Q>
hipError_t launch_decode_mfma_pq(const GroupArgs &ga, int tt, int rt, hipStream_t stream)
{
    if constexpr (activation_field_form(P)) {  // one or two token tiles
        if (tt > 2) return hipErrorInvalidValue;
        if (rt == 2) return tt == 1 ? launch_decode_mfma_v<P, Q, 1, 2>(ga, stream) : launch_decode_mfma_v<P, Q, 2, 2>(ga, stream);
        return tt == 1 ? launch_decode_mfma_v<P, Q, 1, 1>(ga, stream) : launch_decode_mfma_v<P, Q, 2, 1>(ga, stream);
    } else {
        if (rt == 2) {
            if (tt == 1) return launch_decode_mfma_v<P, Q, 1, 2>(ga, stream);
            if (tt == 2) return launch_decode_mfma_v<P, Q, 2, 2>(ga, stream);
            return launch_decode_mfma_v<P, Q, 4, 2>(ga, stream);
        }
        if (tt == 1) return launch_decode_mfma_v<P, Q, 1, 1>(ga, stream);
        if (tt == 2) return launch_decode_mfma_v<P, Q, 2, 1>(ga, stream);
        return launch_decode_mfma_v<P, Q, 4, 1>(ga, stream);
    }
}

hipError_t launch_decode_mfma(const GroupArgs &ga, int rt, hipStream_t stream)
{
    const int p = ga.g[0].p, q = ga.g[0].q, tt = decode_token_tiles(ga.g[0]);
    if (p == 1 && q == 1) return launch_decode_mfma_pq<1, 1>(ga, tt, rt, stream);
    if (p == 1 && q == 2) return launch_decode_mfma_pq<1, 2>(ga, tt, rt, stream);
    if (p == 2 && q == 1) return launch_decode_mfma_pq<2, 1>(ga, tt, rt, stream);
    if (p == 2 && q == 2) return launch_decode_mfma_pq<2, 2>(ga, tt, rt, stream);
    if (p == 3 && q == 1) return launch_decode_mfma_pq<3, 1>(ga, tt, rt, stream);
    if (p == 3 && q == 2) return launch_decode_mfma_pq<3, 2>(ga, tt, rt, stream);
    if (p == 4 && q == 1) return launch_decode_mfma_pq<4, 1>(ga, tt, rt, stream);
    if (p == 4 && q == 2) return launch_decode_mfma_pq<4, 2>(ga, tt, rt, stream);
    // weights of two plane groups (packed activations only)
    if (q == 3) return p == 1 ? launch_decode_mfma_pq<1, 3>(ga, tt, rt, stream) : p == 2 ? launch_decode_mfma_pq<2, 3>(ga, tt, rt, stream)
                     : p == 3 ? launch_decode_mfma_pq<3, 3>(ga, tt, rt, stream) : launch_decode_mfma_pq<4, 3>(ga, tt, rt, stream);
    return p == 1 ? launch_decode_mfma_pq<1, 4>(ga, tt, rt, stream) : p == 2 ? launch_decode_mfma_pq<2, 4>(ga, tt, rt, stream)
         : p == 3 ? launch_decode_mfma_pq<3, 4>(ga, tt, rt, stream) : launch_decode_mfma_pq<4, 4>(ga, tt, rt, stream);
}

// kernel variant that serves a problem: 0 = none, 100 + token tiles = matrix unit, else the token tile of the
// XOR/popcount kernel
int decode_variant(const GemmArgs &g, bool xor_only = false)
{
    if (g.M < 1 || g.M > 64 || g.q < 1 || g.q > 4) return 0;
    if (!xor_only && decode_mfma_supported(g)) return 100 + decode_token_tiles(g);
    if (activation_field_form(g.p)) return 0;  // the XOR/popcount kernel reads the group form only
    if (g.M > 16) return 0;
    return decode_pass_kb(g, decode_mt(g.M)) > 0 ? decode_mt(g.M) : 0;
}

}  // namespace

// M <= 16 with q <= 4, or M <= 64 with p, q <= 2; never activations in the field form (p = 3, 4).
bool gemm_decode_supported(const GemmArgs &g) { return decode_variant(g) != 0; }
bool gemm_decode_valu_supported(const GemmArgs &g) { return decode_variant(g, true) != 0; }

bool gemm_decode_group_supported(const GemmArgs *gs, int count)
{
    if (count < 1 || count > kMaxGroup) return false;
    const int v = decode_variant(gs[0]);
    for (int i = 0; i < count; ++i)
        if (decode_variant(gs[i]) != v || gs[i].p != gs[0].p || gs[i].q != gs[0].q ||
            (gs[i].a_codes != nullptr) != (gs[0].a_codes != nullptr) ||
            (count > 1 && v > 100 && decode_token_groups(gs[i]) > 1))  // token groups: single-problem launches only
            return false;
    return v != 0;
}

hipError_t launch_gemm_decode_group(const GemmArgs *problems, int count, hipStream_t stream, bool xor_only)
{
    GroupArgs ga;
    if (xor_only ? (count != 1 || !gemm_decode_valu_supported(problems[0])) : !gemm_decode_group_supported(problems, count))
        return hipErrorInvalidValue;
    // The workgroups of a launch start in the order of the problems: the problems with the longest K (the
    // longest-running workgroups) go first, so that the launch does not end on them (the seven linears of a
    // Llama-2-7B layer in one launch, 1 / 16 tokens: 14.4 -> 13.4 / 15.4 -> 14.1 us when the down projection, K = 11008,
    // leads instead of trailing).
    GemmArgs gs[kMaxGroup];
    for (int i = 0; i < count; ++i) gs[i] = problems[i];
    std::stable_sort(gs, gs + count, [](const GemmArgs &x, const GemmArgs &y) { return x.nkb > y.nkb; });
    const int variant = decode_variant(gs[0], xor_only);
    if (variant > 100) {
        // two row tiles per workgroup once that still leaves two workgroups per CU
        int64_t rows = 0;
        for (int i = 0; i < count; ++i) rows += gs[i].N;
        // (from unpacked codes already at half as many channels: every workgroup regroups all the codes for itself,
        // so fewer, larger workgroups pay: 7.7 -> 6.7 us for 4 tokens at 11008 x 4096, a loss at 4096 channels)
        int rt = rows >= (gs[0].a_codes ? 256 * 2 * kRowsPerWg : 2 * 256 * 2 * kRowsPerWg) ? 2 : 1;
        if (gs[0].a_codes) {
            // at most two tokens from codes: that kernel variant fits three workgroups per CU
            bool two = true;
            for (int i = 0; i < count; ++i) two = two && gs[i].M <= 2;
            if (two) rt = rows > 3 * 256 * kRowsPerWg ? 2 : 1;
        }
        // four token tiles (33 - 64 tokens) with packed operands: that variant fits one workgroup per CU, so two row
        // tiles as soon as single ones would need a second round of workgroups (8192 x 4096, 64 tokens: 5.9 us)
        if (!gs[0].a_codes && variant == 104 && rows > 256 * kRowsPerWg) rt = 2;
        // packed 3- and 4-bit activations: 88 registers leave two workgroups per CU, so two channel tiles as soon as single
        // ones would need a second round of workgroups (W2A4, one token at 11008 x 4096, cold weights: 7.4 us with single tiles)
        // (with weights of two plane groups the two-tile variant holds too many raw words: 8.8 against 8.2 us for W4A4)
        if (!gs[0].a_codes && activation_field_form(gs[0].p) && gs[0].q <= 2 && rows > 2 * 256 * kRowsPerWg) rt = 2;
        if (gs[0].a_codes && variant == 104) rt = 1;  // four token tiles from codes: two row tiles do not fit the registers
        // weights of two plane groups from codes: the two-tile variant fits three waves per SIMD only (11008 x 4096, 4 / 16
        // tokens: 7.8 / 9.4 us against 6.3 / 7.9 us with single tiles)
        if (gs[0].a_codes && (gs[0].q > 2 || activation_field_form(gs[0].p))) rt = 1;  // (field-form codes: single tiles only)
        if (!make_group(gs, count, kRowsPerWg * rt, [](const GemmArgs &g) { return g.nkb; }, ga))
            return hipErrorInvalidValue;
        return launch_decode_mfma(ga, rt, stream);
    }
    if (!make_group(gs, count, kRowsPerWg, [variant](const GemmArgs &g) { return decode_pass_kb(g, variant); }, ga))
        return hipErrorInvalidValue;
    switch (variant) {
    case 1: return launch_mt<1>(ga, stream);
    case 2: return launch_mt<2>(ga, stream);
    case 4: return launch_mt<4>(ga, stream);
    case 8: return launch_mt<8>(ga, stream);
    default: return launch_mt<16>(ga, stream);
    }
}

hipError_t launch_gemm_decode(const GemmArgs &g, hipStream_t stream) { return launch_gemm_decode_group(&g, 1, stream, false); }
hipError_t launch_gemm_decode_valu(const GemmArgs &g, hipStream_t stream) { return launch_gemm_decode_group(&g, 1, stream, true); }


}  // namespace apmm
