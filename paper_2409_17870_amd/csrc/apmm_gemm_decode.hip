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

#include "apmm_mfma_common.h"

namespace apmm {
namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRowsPerWg = 16;
constexpr int kMaxLdsBytes = 128 * 1024;

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
// Small-M kernel on the matrix unit (3 <= M <= 64, p, q <= 2).  With more than a couple of tokens
// the XOR/popcount form needs 2 p q M lane-operations per weight word and becomes VALU bound; the
// E2M1 MFMA needs one expansion of the weight words (1.25 - 1.5 operations per 8 codes) whatever M is.
// Same split of the work (8 waves over K, lane = weight row l % 16 and k block l / 16 of four), same
// algebra as the large-M MFMA kernel:
//   v_mfma_scale_f32_16x16x128_f8f6f4: A = 16 weight rows x 128 k, B = 128 k x 16 tokens, codes as E2M1;
//   MFMA ks of an iteration multiplies k step ks of the four k blocks held by the four lane groups;
//   a workgroup owns RT tiles of 16 output channels and all TT tiles of 16 tokens: a weight fragment is
//   expanded once and multiplied with TT token fragments, a token fragment with RT weight fragments;
//   the packed activations of all K are copied once per workgroup into LDS as they are, [k block][token][slot],
//   and expanded where they are used; C = acc - 2 cw PA[m] - 2 ca PW[n] + K ca cw with the packed row sums
//   (the operand scales make acc = 4 S).
// RT = 2 halves the number of workgroups (and of activation copies) when there are plenty of output channels.
// ---------------------------------------------------------------------------------------------
template <int P, int Q, int TT, int RT, bool CODES>
__global__ __launch_bounds__(kThreads) void gemm_decode_mfma_kernel(GroupArgs ga)
{
    // which problem of the launch this workgroup works on (uniform over the workgroup); problem 0 from fixed
    // kernel-argument offsets (see gemm_decode_kernel)
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
    static_assert(P <= 2 && Q <= 2, "one plane group per operand");
    constexpr int TOKENS = 16 * TT, ROWS = kRowsPerWg * RT;
    constexpr int OUTS = (TT * RT * 256 + kThreads - 1) / kThreads;  // outputs per thread
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    extern __shared__ __align__(16) uint8_t lds_raw[];
    uint4 *a_lds = reinterpret_cast<uint4 *>(lds_raw);  // [kb][token < TOKENS][slot < P]: packed words as they are
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n0 = (int64_t)block * ROWS;
    constexpr int kSlotVec = kPlaneWords / 4;

    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t rows_b = round_up(g.N, kRowBlock);
    int64_t n_ld[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) n_ld[rt] = n0 + rt * 16 + r16 < rows_b ? n0 + rt * 16 + r16 : rows_b - 1;

    // Order of the requests (see gemm_decode_kernel): this thread's first two vectors of packed activations, then
    // the weights of the first k block, then what only the final store needs.
    const int64_t rows_a = round_up(g.M, kRowBlock);
    const uint32_t vecs_pass0 = (uint32_t)(chunk_kb < g.nkb ? chunk_kb : g.nkb) * P * TOKENS;
    // vector c of a pass that starts at k block kb0 is (k block, slot, token); LDS index = c with slot and token swapped
    auto vec_src = [&](uint32_t c, int64_t kb0, uint32_t &lds_index) {
        const uint32_t m = c % TOKENS, s = (c / TOKENS) % P, ckb = (c / TOKENS) / P;
        const int64_t m_ld = m < rows_a ? m : rows_a - 1;  // tokens past the padded rows are clamped and never stored
        lds_index = (ckb * TOKENS + m) * P + s;
        return reinterpret_cast<const uint4 *>(g.a + tile_row_word(m_ld, kb0 + ckb, g.nkb, P, s));
    };
    constexpr int PEEL = 2;
    uint4 a_first[PEEL];
    uint32_t a_first_index[PEEL];
    if constexpr (!CODES) {
#pragma unroll
        for (int i = 0; i < PEEL; ++i) {
            a_first[i] = make_uint4(0, 0, 0, 0);
            a_first_index[i] = 0;
            if ((uint32_t)tid + i * kThreads < vecs_pass0) a_first[i] = *vec_src(tid + i * kThreads, 0, a_first_index[i]);
        }
    }

    // (from here to the LDS writes every thread issues every load, from clamped addresses where it has nothing
    // to load, see gemm_decode_kernel)
    int64_t kb4 = wave;
    uint4 wnext[RT][2];
    {
        const int64_t kb_ld = kb4 * 4 < g.nkb ? kb4 * 4 + kq : g.nkb - 4 + kq;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const uint4 *wsrc = reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld[rt], kb_ld, g.nkb, Q, 0));
#pragma unroll
            for (int s = 0; s < Q; ++s) wnext[rt][s] = wsrc[s * kSlotVec];
        }
    }

    // What the final store needs is requested now as well and kept as loaded (see gemm_decode_kernel): code sums
    // PA[m], PW[n] and the scales.  Output o of this thread is element (tile t = (tid + o * kThreads) / 256,
    // register v, lane l) of the accumulators, t = rt * TT + tt; 16x16 accumulator layout: lane l, register v holds
    // row 4*(l/16) + v (weight row), column l%16 (token).
    bool out_ok[OUTS];
    int out_m[OUTS];
    int64_t out_n[OUTS];
    uint32_t out_sa_bits[OUTS], out_sw_bits[OUTS], out_pa[OUTS], out_pw[OUTS];
#pragma unroll
    for (int o = 0; o < OUTS; ++o) {
        const int e = tid + o * kThreads, t = e >> 8, v = (e >> 6) & 3, l = e & 63;
        out_m[o] = (t % TT) * 16 + (l & 15);
        out_n[o] = n0 + (t / TT) * 16 + 4 * (l >> 4) + v;
        out_ok[o] = t < TT * RT && out_m[o] < g.M && out_n[o] < g.N;
        // clamped to the padded rows of the sums and to the last entry of the scales; a missing scale vector reads
        // a weight word instead (replaced by 1.0 at the end)
        const int64_t m_c = out_m[o] < rows_a ? out_m[o] : rows_a - 1, n_c = out_n[o] < rows_b ? out_n[o] : rows_b - 1;
        const uint16_t *dummy = reinterpret_cast<const uint16_t *>(g.w);
        // (with activation codes as input the row sum PA[m] is taken while packing, see below)
        out_pa[o] = 0;
        if constexpr (!CODES) out_pa[o] = (uint32_t)g.a_sum[m_c];
        out_pw[o] = (uint32_t)g.w_sum[n_c];
        out_sa_bits[o] = *(g.a_scale ? g.a_scale + (m_c < g.M ? m_c : g.M - 1) : dummy);
        out_sw_bits[o] = *(g.w_scale ? g.w_scale + (n_c < g.N ? n_c : g.N - 1) : dummy);
    }

    mfma::v4f acc[RT][TT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma::v4f{0.f, 0.f, 0.f, 0.f};

    // The activations of chunk_kb k blocks at a time sit in LDS (all of K when it fits, the usual case); a pass
    // boundary is a multiple of 32 k blocks, the stride of the waves' groups of four k blocks.
    uint32_t *pa_lds = reinterpret_cast<uint32_t *>(lds_raw) + chunk_kb * TOKENS * P * 4;  // behind the words
    if constexpr (CODES) {
        if (tid < TOKENS) pa_lds[tid] = 0u;  // token code sums, taken while packing (made visible by the barriers below)
    }
    for (int64_t kb0 = 0; kb0 < g.nkb; kb0 += chunk_kb) {
        const int64_t kb_end = kb0 + chunk_kb < g.nkb ? kb0 + chunk_kb : g.nkb;
        const int64_t pass_kb = kb_end - kb0;
        __syncthreads();  // every wave is done with the previous pass (first pass: the sums are zero)
        if constexpr (CODES) {
            // Straight from the codes: a thread takes the 128 codes of (token m, k block), writes them as the packed
            // words of that row and block (apmm_layout.h) and adds them to the token's code sum.
            const uint32_t total_blocks = (uint32_t)pass_kb * TOKENS;
            for (uint32_t c = tid; c < total_blocks; c += kThreads) {  // consecutive lanes: consecutive 128 bytes of a row
                const uint32_t m = c / (uint32_t)pass_kb, ckb = c - m * (uint32_t)pass_kb;
                uint32_t d[32];
                load_code_block(g.a_codes, g.M, g.K, P, m, kb0 + ckb, d);
                uint32_t sum = 0;
#pragma unroll
                for (int i = 0; i < 32; ++i) sum = __builtin_amdgcn_sad_u8(d[i], 0u, sum);
                // a pass has a multiple of 4 k blocks: the four lanes of an aligned quad hold blocks of the same token
                sum += __shfl_xor(sum, 1);
                sum += __shfl_xor(sum, 2);
                if ((lane & 3) == 0) atomicAdd(&pa_lds[m], sum);
                uint4 *dst = a_lds + (ckb * TOKENS + m) * P;
                if (P == 2) {
                    uint32_t word[8];  // S[w], w = 2 ks + tp: bit b of element (ks, t = 2 tp + tt, jh, c) at 8c + 4jh + 2tt + b
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        word[w] = 0;
#pragma unroll
                        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                            for (int jh = 0; jh < 2; ++jh)
                                word[w] |= d[8 * (w >> 1) + 2 * (2 * (w & 1) + tt) + jh] << (4 * jh + 2 * tt);
                    }
                    dst[0] = make_uint4(word[0], word[1], word[2], word[3]);
                    dst[1] = make_uint4(word[4], word[5], word[6], word[7]);
                } else {
                    uint32_t word[4];  // L[t]: the bit of element (ks, t, jh, c) at 8c + 4jh + ks
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        word[t] = 0;
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks)
                            word[t] |= (d[8 * ks + 2 * t] | (d[8 * ks + 2 * t + 1] << 4)) << ks;
                    }
                    dst[0] = make_uint4(word[0], word[1], word[2], word[3]);
                }
            }
        } else {
            // 16 tokens of a slot are 256 contiguous bytes (tokens past M: the last padded row block holds zero
            // words up to a multiple of 32)
            const uint32_t total_vecs = (uint32_t)pass_kb * P * TOKENS;
            uint32_t c = tid;
            if (kb0 == 0) {  // the vectors requested at the top
#pragma unroll
                for (int i = 0; i < PEEL; ++i)
                    if (c + i * kThreads < total_vecs) a_lds[a_first_index[i]] = a_first[i];
                c += PEEL * kThreads;
            }
            for (; c < total_vecs; c += kThreads) {
                uint32_t index;
                const uint4 v = *vec_src(c, kb0, index);
                a_lds[index] = v;
            }
        }
        __syncthreads();
        if constexpr (CODES) {
            if (kb_end == g.nkb) {  // the code sums are complete
#pragma unroll
                for (int o = 0; o < OUTS; ++o)
                    if (out_ok[o]) out_pa[o] = pa_lds[out_m[o]];
            }
        }

        // nkb and the pass boundaries are multiples of 4: whole groups of four k blocks
        for (; kb4 * 4 < kb_end; kb4 += kWaves) {
            const int64_t kb = kb4 * 4 + kq;
            uint4 wq[RT][2], aq[TT][2];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int s = 0; s < Q; ++s) wq[rt][s] = wnext[rt][s];
            if ((kb4 + kWaves) * 4 < g.nkb) {  // next block of this lane
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const uint4 *wsrc =
                        reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld[rt], kb + 4 * kWaves, g.nkb, Q, 0));
#pragma unroll
                    for (int s = 0; s < Q; ++s) wnext[rt][s] = wsrc[s * kSlotVec];
                }
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int s = 0; s < P; ++s) aq[tt][s] = a_lds[((kb - kb0) * TOKENS + tt * 16 + r16) * P + s];
            mfma::static_for<4>([&](auto ks_c) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_c)::value;
                mfma::v8i a8[RT], b8[TT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) a8[rt] = mfma::v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) b8[tt] = mfma::v8i{0, 0, 0, 0, 0, 0, 0, 0};
                mfma::static_for<4>([&](auto d_c) __attribute__((always_inline)) {
                    constexpr int d = decltype(d_c)::value;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        if constexpr (Q == 1) a8[rt][d] = (int)mfma::fp4_single_dword<ks, d>(wq[rt][0]);
                        else a8[rt][d] = (int)mfma::fp4_pair_dword<ks, d>(wq[rt][0], wq[rt][1]);
                    }
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        if constexpr (P == 1) b8[tt][d] = (int)mfma::fp4_single_dword<ks, d>(aq[tt][0]);
                        else b8[tt][d] = (int)mfma::fp4_pair_dword<ks, d>(aq[tt][0], aq[tt][1]);
                    }
                });
                // E8M0 exponents: 2^2 per operand turns (ua/2)(uw/2) into 4 ua uw
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        acc[rt][tt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                            a8[rt], b8[tt], acc[rt][tt], 4, 4, 0, 129 + (Q == 1 ? mfma::fp4_single_exponent(ks) : 0), 0,
                            129 + (P == 1 ? mfma::fp4_single_exponent(ks) : 0));
            });
        }
    }

    // reduce over the waves through LDS: part[wave][tile t][v][lane]
    __syncthreads();  // every wave is done reading the activations
    float *part = reinterpret_cast<float *>(lds_raw);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[((wave * RT * TT + rt * TT + tt) * 4 + v) * 64 + lane] = acc[rt][tt][v];
    __syncthreads();
#pragma unroll
    for (int o = 0; o < OUTS; ++o) {
        if (!out_ok[o]) continue;
        const int e = tid + o * kThreads;  // = (t * 4 + v) * 64 + l
        float s = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < kWaves; ++w8) s += part[w8 * RT * TT * 256 + e];
        // C = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw
        const uint32_t terms = (uint32_t)g.K * ca * cw - 2u * cw * use_here(out_pa[o]) - 2u * ca * use_here(out_pw[o]);
        const uint32_t sa_bits = g.a_scale ? use_here(out_sa_bits[o]) : 0x3c00u;  // 1.0
        const uint32_t sw_bits = g.w_scale ? use_here(out_sw_bits[o]) : 0x3c00u;
        store_output(g, out_m[o], out_n[o], (int32_t)((uint32_t)(int32_t)s + terms), half_bits_to_float((uint16_t)sa_bits),
                     half_bits_to_float((uint16_t)sw_bits));
    }
}

int decode_token_tiles(int64_t M) { return M <= 16 ? 1 : M <= 32 ? 2 : 4; }

int64_t decode_mfma_pass_kb(const GemmArgs &g)
{
    const int tt = decode_token_tiles(g.M);
    return pass_k_blocks(g.nkb, (size_t)16 * tt * 16 * g.p, (size_t)16 * tt * 4);
}

size_t decode_mfma_lds_bytes(const GemmArgs &g, int rt)
{
    const int tt = decode_token_tiles(g.M);
    const size_t a_bytes = (size_t)decode_mfma_pass_kb(g) * 16 * tt * 16 * g.p + 16 * tt * 4;  // packed words + code sums
    const size_t part_bytes = (size_t)kWaves * rt * tt * 256 * 4;
    return a_bytes > part_bytes ? a_bytes : part_bytes;
}

bool decode_mfma_supported(const GemmArgs &g)
{
    return g.M >= 3 && g.M <= 64 && g.p <= 2 && g.q <= 2 && decode_mfma_pass_kb(g) > 0 &&
           4 * g.nkb * kKBlock * 9 < (1 << 24);
}

template <int P, int Q, int TT, int RT>
hipError_t launch_decode_mfma_v(const GroupArgs &ga, hipStream_t stream)
{
    size_t lds = 0;
    for (int i = 0; i < ga.count; ++i)
        lds = lds > decode_mfma_lds_bytes(ga.g[i], RT) ? lds : decode_mfma_lds_bytes(ga.g[i], RT);
    static bool attr_set[2] = {false, false};
    note_kernel("gemm_decode_mfma_kernel<%d,%d,%d,%d,%s>", P, Q, TT, RT, ga.g[0].a_codes ? "codes" : "packed");
    if (ga.g[0].a_codes) return launch_group(gemm_decode_mfma_kernel<P, Q, TT, RT, true>, attr_set[1], ga, lds, stream);
    return launch_group(gemm_decode_mfma_kernel<P, Q, TT, RT, false>, attr_set[0], ga, lds, stream);
}

template <int P, int Q>
hipError_t launch_decode_mfma_pq(const GroupArgs &ga, int tt, int rt, hipStream_t stream)
{
    if (rt == 2) {
        if (tt == 1) return launch_decode_mfma_v<P, Q, 1, 2>(ga, stream);
        if (tt == 2) return launch_decode_mfma_v<P, Q, 2, 2>(ga, stream);
        return launch_decode_mfma_v<P, Q, 4, 2>(ga, stream);
    }
    if (tt == 1) return launch_decode_mfma_v<P, Q, 1, 1>(ga, stream);
    if (tt == 2) return launch_decode_mfma_v<P, Q, 2, 1>(ga, stream);
    return launch_decode_mfma_v<P, Q, 4, 1>(ga, stream);
}

hipError_t launch_decode_mfma(const GroupArgs &ga, int rt, hipStream_t stream)
{
    const int p = ga.g[0].p, q = ga.g[0].q, tt = decode_token_tiles(ga.g[0].M);
    if (p == 1 && q == 1) return launch_decode_mfma_pq<1, 1>(ga, tt, rt, stream);
    if (p == 1 && q == 2) return launch_decode_mfma_pq<1, 2>(ga, tt, rt, stream);
    if (p == 2 && q == 1) return launch_decode_mfma_pq<2, 1>(ga, tt, rt, stream);
    return launch_decode_mfma_pq<2, 2>(ga, tt, rt, stream);
}

// kernel variant that serves a problem: 0 = none, 100 + token tiles = matrix unit, else the token tile of the
// XOR/popcount kernel
int decode_variant(const GemmArgs &g)
{
    if (g.M < 1 || g.M > 64 || g.q < 1 || g.q > 4) return 0;
    if (activation_field_form(g.p)) return 0;  // 3- and 4-bit activations are laid out for the large-tile MFMA kernel
    if (decode_mfma_supported(g)) return 100 + decode_token_tiles(g.M);
    if (g.M > 16) return 0;
    return decode_pass_kb(g, decode_mt(g.M)) > 0 ? decode_mt(g.M) : 0;
}

}  // namespace

// M <= 16 with q <= 4, or M <= 64 with p, q <= 2; never activations in the field form (p = 3, 4).
bool gemm_decode_supported(const GemmArgs &g) { return decode_variant(g) != 0; }

bool gemm_decode_group_supported(const GemmArgs *gs, int count)
{
    if (count < 1 || count > kMaxGroup) return false;
    const int v = decode_variant(gs[0]);
    for (int i = 0; i < count; ++i)
        if (decode_variant(gs[i]) != v || gs[i].p != gs[0].p || gs[i].q != gs[0].q ||
            (gs[i].a_codes != nullptr) != (gs[0].a_codes != nullptr))
            return false;
    return v != 0;
}

hipError_t launch_gemm_decode_group(const GemmArgs *gs, int count, hipStream_t stream)
{
    GroupArgs ga;
    if (!gemm_decode_group_supported(gs, count)) return hipErrorInvalidValue;
    const int variant = decode_variant(gs[0]);
    if (variant > 100) {
        // two row tiles per workgroup once that still leaves two workgroups per CU
        int64_t rows = 0;
        for (int i = 0; i < count; ++i) rows += gs[i].N;
        // (from unpacked codes already at half as many channels: every workgroup regroups all the codes for itself,
        // so fewer, larger workgroups pay: 7.7 -> 6.7 us for 4 tokens at 11008 x 4096, a loss at 4096 channels)
        const int rt = rows >= (gs[0].a_codes ? 256 * 2 * kRowsPerWg : 2 * 256 * 2 * kRowsPerWg) ? 2 : 1;
        if (!make_group(gs, count, kRowsPerWg * rt, [](const GemmArgs &g) { return decode_mfma_pass_kb(g); }, ga))
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

hipError_t launch_gemm_decode(const GemmArgs &g, hipStream_t stream) { return launch_gemm_decode_group(&g, 1, stream); }


}  // namespace apmm
