// Design A: bit planes recombined into int8 on chip, int8 MFMA, int32 accumulate.
//
// Paper Sec. 3.2 recovers C = sum_i sum_j 2^(i+j) * D_ij from p*q one-bit products.  The
// matrix unit of gfx950 multiplies int8, not single bits, so the shift-and-add is moved in
// front of the multiplier: the planes of each operand are combined into the int8 value
//   v = sum_i (2*b_i - 1) * 2^i                                   (paper Eq. 1)
// while the tile is copied from registers to LDS, and ONE int8 MFMA pass produces
// sum_k a_k * w_k = sum_ij 2^(i+j) D_ij directly.  This is the recovery of paper Sec. 4.2
// done entirely in registers/LDS (nothing but C reaches global memory), at the cost of one
// MFMA pass instead of p*q.
//
// Workgroup = 256 threads = 2 x 2 waves; wave tile (32*WM) x (32*WN), workgroup tile
// BM x BN = (64*WM) x (64*WN); k step 128 (one packed tile per row block).
// Per k step (paper Sec. 4.2, items 2 and 3: K partition and ping-pong buffers):
//   global -> registers : packed plane words of the NEXT k block (P + Q words per row and 32 k)
//   registers -> LDS    : expand to int8 in the MFMA operand order, into the idle LDS buffer
//   LDS -> MFMA         : ds_read_b128 fragments of the current buffer, v_mfma_i32_32x32x32_i8
//
// LDS tile layout of one operand and stage: [ks = 4][row block][half = 2][row = 32][16 bytes],
// i.e. the 1 KB fragment of one MFMA (32 rows x 32 k) is contiguous and lane l reads bytes
// 16*l .. 16*l+15: conflict free for ds_read_b128 and for the ds_write_b128 of the expansion.
// The k order inside a fragment is (half, byte) = the order the expansion produces; both
// operands use the same order, which is all the contraction needs.
#include "apmm_epilogue.h"
#include "apmm_kernels.h"

namespace apmm {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kStageK = 128;  // k elements per LDS stage (= one packed k block)

// Planes w[0..NB-1] of one 32-element group -> 8 dwords of int8 values (elements 4t..4t+3 in dword t).
// Two's-complement byte of v = 2u + 1 - 2^NB: collect x = 2u per byte (plane i to bit i+1), then
// (x + (0x80 - 2^NB)) ^ 0x81; the sum stays below 0x100 for NB <= 7, so bytes never interact.
template <int NB>
__device__ __forceinline__ void expand_group(const uint32_t (&w)[NB], uint32_t (&out)[8])
{
    constexpr uint32_t bias = (uint32_t)(0x80 - (1 << NB)) * 0x01010101u;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint32_t x = 0;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int sh = t - (i + 1);
            const uint32_t s = (sh >= 0) ? (w[i] >> sh) : (w[i] << (-sh));
            x |= s & (0x01010101u << (i + 1));
        }
        out[t] = (x + bias) ^ 0x81818181u;
    }
}

template <int NB, int WX>
struct Loader {
    static constexpr int BX = 64 * WX;  // rows of the workgroup tile
    uint32_t regs[WX][NB];
    const uint32_t *src[WX];  // word address of (row, plane 0, word gq) in k block 0
    int lds_off[WX];          // byte offset of the unit's first 16-byte chunk inside the operand stage

    __device__ __forceinline__ void init(const uint32_t *packed, int64_t row0, int64_t rows_p, int64_t nkb,
                                         int tid)
    {
#pragma unroll
        for (int s = 0; s < WX; ++s) {
            const int u = tid + kThreads * s;
            const int row = u % BX, gq = u / BX;
            int64_t grow = row0 + row;
            if (grow >= rows_p) grow = rows_p - 1;  // rows past the operand: read a valid row, never stored
            src[s] = packed + tile_row_word(grow, 0, nkb, NB, 0) + gq;
            lds_off[s] = ((gq * (BX / 32) + row / 32) * 2) * 512 + (row % 32) * 16;
        }
    }
    __device__ __forceinline__ void fetch(int64_t kb)
    {
#pragma unroll
        for (int s = 0; s < WX; ++s)
#pragma unroll
            for (int i = 0; i < NB; ++i)
                regs[s][i] = src[s][kb * (kRowBlock * kWordsPerRow * NB) + i * kWordsPerRow];
    }
    __device__ __forceinline__ void expand_to_lds(uint8_t *stage) const
    {
#pragma unroll
        for (int s = 0; s < WX; ++s) {
            uint32_t o[8];
            expand_group<NB>(regs[s], o);
            uint4 *dst = reinterpret_cast<uint4 *>(stage + lds_off[s]);
            dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
            dst[32] = make_uint4(o[4], o[5], o[6], o[7]);  // second half: +512 bytes
        }
    }
};

template <int P, int Q, int WM, int WN>
__global__ __launch_bounds__(kThreads) void gemm_mfma_kernel(GemmArgs g, int tiles_n, int tiles_total)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int A_STAGE = BM * kStageK, B_STAGE = BN * kStageK;  // bytes of int8
    extern __shared__ __align__(16) uint8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
    // tiles so that the packed rows it re-reads stay in its own L2.
    int lid = blockIdx.x;
    if ((tiles_total & 7) == 0) lid = (blockIdx.x & 7) * (tiles_total >> 3) + (blockIdx.x >> 3);
    const int tm = lid / tiles_n, tn = lid % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    Loader<P, WM> la;
    Loader<Q, WN> lb;
    la.init(g.a, m0, round_up(g.M, kRowBlock), g.nkb, tid);
    lb.init(g.w, n0, round_up(g.N, kRowBlock), g.nkb, tid);

    v16i acc[WM][WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi)
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0;

    la.fetch(0);
    lb.fetch(0);
    la.expand_to_lds(lds);
    lb.expand_to_lds(lds + A_STAGE);
    __syncthreads();

    for (int64_t kb = 0; kb < g.nkb; ++kb) {
        const uint8_t *cur = lds + (kb & 1) * (A_STAGE + B_STAGE);
        uint8_t *nxt = lds + ((kb + 1) & 1) * (A_STAGE + B_STAGE);
        const bool more = kb + 1 < g.nkb;
        if (more) {
            la.fetch(kb + 1);
            lb.fetch(kb + 1);
        }
        const uint8_t *fa = cur + (wave_m * WM) * 1024 + lane * 16;
        const uint8_t *fb = cur + A_STAGE + (wave_n * WN) * 1024 + lane * 16;
#pragma unroll
        for (int ks = 0; ks < kStageK / 32; ++ks) {
            v4i af[WM], bf[WN];
#pragma unroll
            for (int bi = 0; bi < WM; ++bi)
                af[bi] = *reinterpret_cast<const v4i *>(fa + (ks * (BM / 32) + bi) * 1024);
#pragma unroll
            for (int bj = 0; bj < WN; ++bj)
                bf[bj] = *reinterpret_cast<const v4i *>(fb + (ks * (BN / 32) + bj) * 1024);
#pragma unroll
            for (int bi = 0; bi < WM; ++bi)
#pragma unroll
                for (int bj = 0; bj < WN; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[bi], bf[bj], acc[bi][bj], 0, 0, 0);
        }
        if (more) {
            la.expand_to_lds(nxt);
            lb.expand_to_lds(nxt + A_STAGE);
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: lane l, register v holds
    //   row = 8*(v/4) + 4*(l/32) + v%4, column = l%32.
    const int col = lane & 31, rsub = (lane >> 5) * 4;
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        const int64_t n = n0 + (wave_n * WN + bj) * 32 + col;
        if (n >= g.N) continue;
        const float sw = load_scale(g.w_scale, n);
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + (wave_m * WM + bi) * 32 + 8 * (v / 4) + rsub + (v % 4);
                if (m >= g.M) continue;
                store_output(g, m, n, acc[bi][bj][v] - g.pad_corr, load_scale(g.a_scale, m), sw);
            }
        }
    }
}

template <int P, int Q, int WM, int WN>
hipError_t launch_variant(const GemmArgs &g, hipStream_t stream)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * kStageK;
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int64_t tiles = tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kernel = gemm_mfma_kernel<P, Q, WM, WN>;
    static bool attr_set = false;  // raising the dynamic LDS limit is idempotent; a race here is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(kThreads), lds_bytes, stream, g, (int)tiles_n,
                       (int)tiles);
    return hipGetLastError();
}

template <int P, int Q>
hipError_t launch_pq(const GemmArgs &g, hipStream_t stream)
{
    const int64_t big = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big >= 192) return launch_variant<P, Q, 4, 4>(g, stream);
    return launch_variant<P, Q, 2, 2>(g, stream);
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs &g) { return g.p >= 1 && g.p <= 4 && g.q >= 1 && g.q <= 4; }

hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t stream)
{
#define APMM_CASE(P_, Q_) \
    if (g.p == P_ && g.q == Q_) return launch_pq<P_, Q_>(g, stream);
    APMM_CASE(1, 1) APMM_CASE(1, 2) APMM_CASE(1, 3) APMM_CASE(1, 4)
    APMM_CASE(2, 1) APMM_CASE(2, 2) APMM_CASE(2, 3) APMM_CASE(2, 4)
    APMM_CASE(3, 1) APMM_CASE(3, 2) APMM_CASE(3, 3) APMM_CASE(3, 4)
    APMM_CASE(4, 1) APMM_CASE(4, 2) APMM_CASE(4, 3) APMM_CASE(4, 4)
#undef APMM_CASE
    return hipErrorInvalidValue;
}

}  // namespace apmm
