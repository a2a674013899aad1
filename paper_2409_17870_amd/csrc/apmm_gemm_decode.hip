// Small-M (decode) kernel, design B: the packed weights are streamed once from HBM and every
// plane pair is multiplied by XOR + popcount on the vector ALU (paper Sec. 3.2 with the XOR form
// of the 1-bit product):
//   D_ij = K - 2 * popcount(a^(j) xor w^(i)),   C = sum_ij 2^(i+j) D_ij
//        = K (2^p - 1)(2^q - 1) - 2 * sum_ij 2^(i+j) popcount(a^(j) xor w^(i)).
// Padded k positions hold equal bits in both operands and drop out of the popcounts.  The
// shift-and-add recovery runs in registers, the reduction over K in registers, DPP-free lane
// shuffles and LDS; only C reaches global memory (paper Sec. 4.2).
//
// Work split.  With M <= 16 tokens the weights (N*K*q/8 bytes) are the only real traffic, a few
// MiB, i.e. a few KiB per CU: the kernel is latency bound, so everything is loaded up front with
// as many waves as possible.
//   workgroup : 16 output channels (half a packed row block), 8 waves
//   wave      : k blocks 4*(w + 8*t) .. +3, t = 0, 1, ...
//   lane l    : weight row l % 16, k block l / 16 of the wave's four; it loads the row's q planes
//               of that block (q x 16 bytes, 256 contiguous bytes per 16 lanes) straight into registers
// The activations (M rows, all K) are copied once per workgroup from their packed tiles into LDS
// with every plane rotated back to the natural bit order; a weight plane is rotated back the same
// way after loading, so that any activation plane can be XOR-ed with any weight plane.
#include "apmm_mfma_common.h"

namespace apmm {
namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRowsPerWg = 16;
constexpr int kMaxLdsBytes = 128 * 1024;

template <int MT, int Q>
__global__ __launch_bounds__(kThreads) void gemm_decode_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    uint4 *a_lds = reinterpret_cast<uint4 *>(lds_raw);  // [kb][m < MT][j < p] natural-order plane words
    const int p = g.p;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * kRowsPerWg;

    // activations -> LDS: chunk (kb, m, j) = 16 bytes of plane j of row m in k block kb
    const int chunks_per_kb = MT * p;
    const int64_t total_chunks = g.nkb * chunks_per_kb;
    for (int64_t c = tid; c < total_chunks; c += kThreads) {
        const int64_t kb = c / chunks_per_kb;
        const int rem = (int)(c % chunks_per_kb), m = rem / p, j = rem % p;
        uint4 v = *reinterpret_cast<const uint4 *>(g.a + tile_row_word(m, kb, g.nkb, p, j));
        const int rot = plane_rotation(j);
        v.x = __builtin_rotateright32(v.x, rot);
        v.y = __builtin_rotateright32(v.y, rot);
        v.z = __builtin_rotateright32(v.z, rot);
        v.w = __builtin_rotateright32(v.w, rot);
        a_lds[c] = v;
    }
    __syncthreads();

    const int row = lane & 15, sub = lane >> 4;
    int64_t n = n0 + row;
    const int64_t n_ld = n < round_up(g.N, kRowBlock) ? n : round_up(g.N, kRowBlock) - 1;

    uint32_t acc[MT];  // sum_ij 2^(i+j) popcount, modulo 2^32
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0;

    for (int64_t kb = 4 * (int64_t)wave + sub; kb < g.nkb; kb += 4 * kWaves) {
        uint4 w[Q];
        const uint4 *wsrc = reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld, kb, g.nkb, Q, 0));
#pragma unroll
        for (int i = 0; i < Q; ++i) w[i] = wsrc[i * (kPlaneWords / 4)];
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            w[i].x = __builtin_rotateright32(w[i].x, plane_rotation(i));
            w[i].y = __builtin_rotateright32(w[i].y, plane_rotation(i));
            w[i].z = __builtin_rotateright32(w[i].z, plane_rotation(i));
            w[i].w = __builtin_rotateright32(w[i].w, plane_rotation(i));
        }
        const uint4 *arow = a_lds + kb * chunks_per_kb;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            for (int j = 0; j < p; ++j) {
                const uint4 a = arow[m * p + j];
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    const uint32_t pc = __popc(a.x ^ w[i].x) + __popc(a.y ^ w[i].y) + __popc(a.z ^ w[i].z) +
                                        __popc(a.w ^ w[i].w);
                    acc[m] += pc << (i + j);
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
    if (tid < MT * kRowsPerWg) {
        const int m = tid / kRowsPerWg, r = tid % kRowsPerWg;
        uint32_t s = 0;
#pragma unroll
        for (int w8 = 0; w8 < kWaves; ++w8) s += part[(w8 * MT + m) * kRowsPerWg + r];
        n = n0 + r;
        if (m < g.M && n < g.N) {
            const uint32_t full = (uint32_t)g.K * (uint32_t)((1 << p) - 1) * (uint32_t)((1 << Q) - 1);
            store_output(g, m, n, (int32_t)(full - 2u * s), load_scale(g.a_scale, m), load_scale(g.w_scale, n));
        }
    }
}

size_t decode_lds_bytes(const GemmArgs &g, int mt)
{
    const size_t a_bytes = (size_t)g.nkb * mt * g.p * 16;
    const size_t part_bytes = (size_t)kWaves * mt * kRowsPerWg * 4;
    return a_bytes > part_bytes ? a_bytes : part_bytes;
}

int decode_mt(int64_t M) { return M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : 16; }

template <int MT, int Q>
hipError_t launch_mt_q(const GemmArgs &g, hipStream_t stream)
{
    const size_t lds = decode_lds_bytes(g, MT);
    auto kernel = gemm_decode_kernel<MT, Q>;
    static bool attr_set = false;  // idempotent; a race here is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t wgs = (g.N + kRowsPerWg - 1) / kRowsPerWg;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(kThreads), lds, stream, g);
    return hipGetLastError();
}

template <int MT>
hipError_t launch_mt(const GemmArgs &g, hipStream_t stream)
{
    switch (g.q) {
    case 1: return launch_mt_q<MT, 1>(g, stream);
    case 2: return launch_mt_q<MT, 2>(g, stream);
    case 3: return launch_mt_q<MT, 3>(g, stream);
    case 4: return launch_mt_q<MT, 4>(g, stream);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Small-M kernel on the matrix unit (3 <= M <= 16, p, q <= 2).  With more than a couple of tokens
// the XOR/popcount form needs 2 p q M lane-operations per weight word and becomes VALU bound; the
// E2M1 MFMA needs one expansion of the weight word (q + 1 operations per 8 codes) whatever M is.
// Same split of the work (16 output channels per workgroup, 8 waves over K, lane = weight row l % 16
// and k block l / 16 of four), same algebra as the large-M MFMA kernels:
//   v_mfma_scale_f32_16x16x128_f8f6f4: A = 16 weight rows x 128 k, B = 128 k x 16 tokens, codes as E2M1;
//   MFMA g of an iteration multiplies word group g of the four k blocks held by the four lane groups;
//   the packed activations of all K are copied once per workgroup into LDS as [k block][word group][token]
//   plane words and expanded where they are used; C = 16 acc - 2 cw PA[m] - 2 ca PW[n] + K ca cw with the packed row sums.
// ---------------------------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));

template <int P, int Q>
__global__ __launch_bounds__(kThreads) void gemm_decode_mfma_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) uint8_t lds_raw[];
    uint32_t *a_lds = reinterpret_cast<uint32_t *>(lds_raw);  // [kb][gq][token < 16][plane]: raw plane words
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * kRowsPerWg;

    // activations -> LDS as they are packed (expanded at use).  One 16-byte load brings the four word
    // groups of (k block, plane, token); 16 tokens are 256 contiguous bytes.
    const int64_t total_vecs = g.nkb * P * 16;
    for (int64_t c = tid; c < total_vecs; c += kThreads) {
        const int m = (int)(c & 15);
        const int i = (int)((c >> 4) % P);
        const int64_t kb = (c >> 4) / P;
        const uint4 v = *reinterpret_cast<const uint4 *>(g.a + tile_row_word(m, kb, g.nkb, P, i));
        uint32_t *dst = a_lds + ((kb * kWordsPerRow) * 16 + m) * P + i;
        dst[0 * 16 * P] = v.x;
        dst[1 * 16 * P] = v.y;
        dst[2 * 16 * P] = v.z;
        dst[3 * 16 * P] = v.w;
    }
    __syncthreads();

    const int r16 = lane & 15, kq = lane >> 4;
    const int64_t rows_b = round_up(g.N, kRowBlock);
    const int64_t n_ld = n0 + r16 < rows_b ? n0 + r16 : rows_b - 1;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    // nkb is a multiple of 4 (K is padded to 512): whole groups of four k blocks
    for (int64_t kb4 = wave; kb4 * 4 < g.nkb; kb4 += kWaves) {
        const int64_t kb = kb4 * 4 + kq;
        uint4 wq[Q];
        const uint4 *wsrc = reinterpret_cast<const uint4 *>(g.w + tile_row_word(n_ld, kb, g.nkb, Q, 0));
#pragma unroll
        for (int i = 0; i < Q; ++i) wq[i] = wsrc[i * (kPlaneWords / 4)];
        const uint32_t *arow = a_lds + ((kb * kWordsPerRow) * 16 + r16) * P;
        mfma::static_for<4>([&](auto g_c) __attribute__((always_inline)) {
            constexpr int gq = decltype(g_c)::value;
            uint32_t w[Q];
#pragma unroll
            for (int i = 0; i < Q; ++i) w[i] = gq == 0 ? wq[i].x : gq == 1 ? wq[i].y : gq == 2 ? wq[i].z : wq[i].w;
            const mfma::v8i a8 = {(int)mfma::expand_dword<Q, true>(w, 0), (int)mfma::expand_dword<Q, true>(w, 1),
                                  (int)mfma::expand_dword<Q, true>(w, 2), (int)mfma::expand_dword<Q, true>(w, 3),
                                  0, 0, 0, 0};
            uint32_t aw[P];
#pragma unroll
            for (int i = 0; i < P; ++i) aw[i] = arow[gq * 16 * P + i];
            const mfma::v8i b8 = {(int)mfma::expand_dword<P, true>(aw, 0), (int)mfma::expand_dword<P, true>(aw, 1),
                                  (int)mfma::expand_dword<P, true>(aw, 2), (int)mfma::expand_dword<P, true>(aw, 3),
                                  0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc, 4, 4, 0, 127, 0, 127);
        });
    }

    // reduce over the waves through LDS: part[wave][v][lane]
    __syncthreads();  // every wave is done reading the activations
    float *part = reinterpret_cast<float *>(lds_raw);
#pragma unroll
    for (int v = 0; v < 4; ++v) part[(wave * 4 + v) * 64 + lane] = acc[v];
    __syncthreads();
    if (tid < 256) {
        const int l = tid & 63, v = tid >> 6;
        float s = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < kWaves; ++w8) s += part[(w8 * 4 + v) * 64 + l];
        // 16x16 accumulator layout: lane l, register v holds row 4*(l/16) + v (weight row), column l%16 (token)
        const int m = l & 15;
        const int64_t n = n0 + 4 * (l >> 4) + v;
        if (m < g.M && n < g.N) {
            constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
            const uint32_t c = (uint32_t)(int32_t)(s * 16.0f) - 2u * cw * (uint32_t)g.a_sum[m] -
                               2u * ca * (uint32_t)g.w_sum[n] + (uint32_t)g.K * ca * cw;
            store_output(g, m, n, (int32_t)c, load_scale(g.a_scale, m), load_scale(g.w_scale, n));
        }
    }
}

size_t decode_mfma_lds_bytes(const GemmArgs &g)
{
    const size_t a_bytes = (size_t)g.nkb * kWordsPerRow * 16 * 4 * g.p;
    const size_t part_bytes = (size_t)kWaves * 4 * 64 * 4;
    return a_bytes > part_bytes ? a_bytes : part_bytes;
}

bool decode_mfma_supported(const GemmArgs &g)
{
    return g.M >= 3 && g.M <= 16 && g.p <= 2 && g.q <= 2 && decode_mfma_lds_bytes(g) <= (size_t)kMaxLdsBytes &&
           g.nkb * kKBlock <= (1 << 18);
}

template <int P, int Q>
hipError_t launch_decode_mfma_pq(const GemmArgs &g, hipStream_t stream)
{
    auto kernel = gemm_decode_mfma_kernel<P, Q>;
    static bool attr_set = false;  // idempotent; a race here is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t wgs = (g.N + kRowsPerWg - 1) / kRowsPerWg;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(kThreads), decode_mfma_lds_bytes(g), stream, g);
    return hipGetLastError();
}

hipError_t launch_decode_mfma(const GemmArgs &g, hipStream_t stream)
{
    if (g.p == 1 && g.q == 1) return launch_decode_mfma_pq<1, 1>(g, stream);
    if (g.p == 1 && g.q == 2) return launch_decode_mfma_pq<1, 2>(g, stream);
    if (g.p == 2 && g.q == 1) return launch_decode_mfma_pq<2, 1>(g, stream);
    return launch_decode_mfma_pq<2, 2>(g, stream);
}

}  // namespace

// M <= 16, q <= 4, and the activations of all K must fit the LDS budget.
bool gemm_decode_supported(const GemmArgs &g)
{
    if (g.M < 1 || g.M > 16 || g.q < 1 || g.q > 4) return false;
    return decode_lds_bytes(g, decode_mt(g.M)) <= (size_t)kMaxLdsBytes;
}

hipError_t launch_gemm_decode(const GemmArgs &g, hipStream_t stream)
{
    if (decode_mfma_supported(g)) return launch_decode_mfma(g, stream);
    switch (decode_mt(g.M)) {
    case 1: return launch_mt<1>(g, stream);
    case 2: return launch_mt<2>(g, stream);
    case 4: return launch_mt<4>(g, stream);
    case 8: return launch_mt<8>(g, stream);
    default: return launch_mt<16>(g, stream);
    }
}

}  // namespace apmm
