// Design A: bit planes recombined into int8 on chip, int8 MFMA, int32 accumulate.
//
// Paper Sec. 3.2 recovers C = sum_i sum_j 2^(i+j) * D_ij from p*q one-bit products.  The
// matrix unit of gfx950 multiplies int8, not single bits, so the shift-and-add is moved in
// front of the multiplier: while the tile is copied from registers to LDS, the planes of
// each operand are combined into the code u = sum_i b_i 2^i as an int8 byte; by paper Eq. 1 the
// value is v = sum_i (2*b_i - 1) * 2^i = 2u - (2^n - 1).  ONE int8 MFMA pass gives
// S = sum_k ua_k * uw_k, and with the row sums of the codes (weighted popcounts of the planes,
// taken by the same threads that expand them)
//   C = sum_k (2 ua_k - ca)(2 uw_k - cw),   ca = 2^p - 1, cw = 2^q - 1
//     = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw,
//   PA[m] = sum_i 2^i * popcount(plane i of row m)  (padded k positions included: they hold the
//   code ca resp. cw in both operands, which is why the true K appears in the constant),
// which equals sum_ij 2^(i+j) D_ij.  This is the recovery of paper Sec. 4.2 done entirely in
// registers/LDS (nothing but C reaches global memory), at the cost of one MFMA pass instead
// of p*q, and the expansion costs one AND(-OR) per plane plus one rotate per four elements.
//
// Workgroup = 256 threads = 2 x 2 waves; wave tile (32*WM) x (32*WN), workgroup tile
// BM x BN = (64*WM) x (64*WN); k step 128 (one packed tile per row block).
// Per k step (paper Sec. 4.2, items 2 and 3: K partition and ping-pong buffers):
//   global -> registers : packed plane words two k blocks ahead (P + Q words per row and 32 k)
//   registers -> LDS    : expand the next k block to int8 in MFMA operand order, into the idle buffer
//   LDS -> MFMA         : ds_read_b128 fragments of the current buffer, v_mfma_i32_32x32x32_i8
// The three activities of one k step sit in one basic block and are interleaved
// instruction by instruction (one MFMA, then its share of expansion VALU work and LDS
// traffic), because a wave owns its SIMD alone (512 registers) and nothing else would
// cover the matrix unit while the VALU expands.
//
// LDS tile layout of one operand and stage: [ks = 4][row block][half = 2][row = 32][16 bytes],
// i.e. the 1 KB fragment of one MFMA (32 rows x 32 k) is contiguous and lane l reads bytes
// 16*l .. 16*l+15: conflict free for ds_read_b128 and for the ds_write_b128 of the expansion.
// The k order inside a fragment is (half, byte) = the order the expansion produces; both
// operands use the same order, which is all the contraction needs.
#pragma once
#include <type_traits>
#include <utility>

#include "apmm_epilogue.h"
#include "apmm_kernels.h"

namespace apmm {
namespace mfma {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kStageK = 128;  // k elements per LDS stage (= one packed k block)

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), always flattened,
// so that every index below is a constant (shift amounts, register numbers, LDS offsets).
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Dword t (elements 4t .. 4t+3) of the int8 expansion of one 32-element group given its planes
// w[0..NB-1]: byte = code u.  Plane i is stored rotated left by i, so its bits for these four
// elements are at in-byte position (t + i) % 8, and one rotate right by t brings every plane to
// its own bit i (apmm_layout.h).
template <int NB>
__device__ __forceinline__ uint32_t expand_dword(const uint32_t (&w)[NB], int t)
{
    uint32_t y = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) y |= w[i] & (0x01010101u << ((t + i) % 8));
    return t ? __builtin_rotateright32(y, t) : y;
}

// Per-thread share of one operand's workgroup tile: WX units, one unit = (row, 32-k word group).
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
    // whole share at once (prologue)
    __device__ __forceinline__ void expand_to_lds(uint8_t *stage, uint32_t (&counts)[NB]) const
    {
        uint32_t o[4];
#pragma unroll
        for (int task = 0; task < 8 * WX; ++task) expand_task(stage, task, o, counts);
    }
    // one dword of the share: task = 8 * unit + t; every fourth task stores 16 bytes to LDS, and the
    // first task of a unit adds the unit's plane popcounts to `counts`
    __device__ __forceinline__ void expand_task(uint8_t *stage, int task, uint32_t (&o)[4],
                                                uint32_t (&counts)[NB]) const
    {
        const int s = task / 8, t = task % 8;
        if (t == 0) {
#pragma unroll
            for (int i = 0; i < NB; ++i) counts[i] += __popc(regs[s][i]);
        }
        o[t % 4] = expand_dword<NB>(regs[s], t);
        if (t % 4 == 3)
            *reinterpret_cast<uint4 *>(stage + lds_off[s] + (t / 4) * 512) = make_uint4(o[0], o[1], o[2], o[3]);
    }
};

template <int P, int Q, int WM, int WN>
__global__ __launch_bounds__(kThreads) void gemm_mfma_kernel(GemmArgs g, int tiles_n, int tiles_total)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int A_STAGE = BM * kStageK, B_STAGE = BN * kStageK;  // bytes of int8
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int KS = kStageK / 32;  // MFMA k steps per stage
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

    const int64_t last = g.nkb - 1;
    la.fetch(0);
    lb.fetch(0);
    // per plane: set bits of this thread's units so far (all units of a thread lie in one row)
    uint32_t pop_a[P], pop_b[Q];
#pragma unroll
    for (int i = 0; i < P; ++i) pop_a[i] = 0;
#pragma unroll
    for (int i = 0; i < Q; ++i) pop_b[i] = 0;
    la.expand_to_lds(lds, pop_a);
    lb.expand_to_lds(lds + A_STAGE, pop_b);
    la.fetch(last < 1 ? last : 1);
    lb.fetch(last < 1 ? last : 1);
    __syncthreads();

    const int frag_a = (wave_m * WM) * 1024 + lane * 16;
    const int frag_b = A_STAGE + (wave_n * WN) * 1024 + lane * 16;

    constexpr int MFMAS = WM * WN * KS;             // MFMAs per stage and wave
    constexpr int PER_KS = WM * WN;                 // MFMAs per 32-k step
    constexpr int READS = WM + WN;                  // fragment reads per 32-k step
    constexpr int TASKS_A = 8 * WM, TASKS = 8 * (WM + WN);  // expansion dwords per thread and stage
    static_assert(TASKS % MFMAS == 0 || MFMAS % TASKS == 0, "expansion tasks must spread evenly over the MFMAs");

    for (int64_t kb = 0; kb < g.nkb; ++kb) {
        const uint8_t *cur = lds + (kb & 1) * STAGE;
        uint8_t *nxt = lds + ((kb + 1) & 1) * STAGE;

        // raw planes of k block kb+1 are in registers; start the loads of kb+2 right away
        Loader<P, WM> ea = la;
        Loader<Q, WN> eb = lb;
        const int64_t kf = (kb + 2 <= last) ? kb + 2 : last;  // clamped: the surplus fetches are discarded
        la.fetch(kf);
        lb.fetch(kf);
        // the last iteration re-expands the final k block: its popcounts must not be counted twice
        uint32_t cnt_a[P], cnt_b[Q];
#pragma unroll
        for (int i = 0; i < P; ++i) cnt_a[i] = 0;
#pragma unroll
        for (int i = 0; i < Q; ++i) cnt_b[i] = 0;

        v4i af[2][WM], bf[2][WN];
        // fragment r of 32-k step ks: r = 0 -> A block 0, r = 1..WN -> B blocks, then the other A blocks
        auto read_frag = [&](auto ks_c, auto r_c) __attribute__((always_inline)) {
            constexpr int ks = decltype(ks_c)::value, r = decltype(r_c)::value;
            if constexpr (r == 0)
                af[ks & 1][0] = *reinterpret_cast<const v4i *>(cur + frag_a + (ks * (BM / 32)) * 1024);
            else if constexpr (r <= WN)
                bf[ks & 1][r - 1] = *reinterpret_cast<const v4i *>(cur + frag_b + (ks * (BN / 32) + r - 1) * 1024);
            else
                af[ks & 1][r - WN] = *reinterpret_cast<const v4i *>(cur + frag_a + (ks * (BM / 32) + r - WN) * 1024);
        };
        static_for<READS>([&](auto r_c) __attribute__((always_inline)) {
            read_frag(std::integral_constant<int, 0>{}, r_c);
        });
        __builtin_amdgcn_sched_barrier(0);

        uint32_t oa[4], ob[4];
        static_for<MFMAS>([&](auto i_c) __attribute__((always_inline)) {
            constexpr int i = decltype(i_c)::value;
            constexpr int ks = i / PER_KS, j = i % PER_KS, bi = j / WN, bj = j % WN;
            // prefetch the fragments of the next 32-k step, spread over this step's MFMAs
            if constexpr (ks + 1 < KS) {
                static_for<READS>([&](auto r_c) __attribute__((always_inline)) {
                    if constexpr (decltype(r_c)::value * PER_KS / READS == j)
                        read_frag(std::integral_constant<int, ks + 1>{}, r_c);
                });
            }
            acc[bi][bj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks & 1][bi], bf[ks & 1][bj], acc[bi][bj], 0, 0, 0);
            // this MFMA's share of the expansion of k block kb+1 into the idle buffer (in the last
            // iteration it rewrites the block already there: harmless, and keeps the body branch free)
            static_for<TASKS>([&](auto t_c) __attribute__((always_inline)) {
                constexpr int task = decltype(t_c)::value;
                if constexpr (task * MFMAS / TASKS == i) {
                    if constexpr (task < TASKS_A)
                        ea.expand_task(nxt, task, oa, cnt_a);
                    else
                        eb.expand_task(nxt + A_STAGE, task - TASKS_A, ob, cnt_b);
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        const uint32_t keep = (kb < last) ? 0xffffffffu : 0u;
#pragma unroll
        for (int i = 0; i < P; ++i) pop_a[i] += cnt_a[i] & keep;
#pragma unroll
        for (int i = 0; i < Q; ++i) pop_b[i] += cnt_b[i] & keep;
        __syncthreads();
    }

    // Row and column terms of the recovery.  A thread's units all lie in row tid % BX of its operand
    // tile; 256 / BX threads share a row, each leaves its partial in LDS (free now: the loop ended
    // with a barrier) and the readers add them up.
    constexpr int SHARE_A = kThreads / BM > 0 ? kThreads / BM : 1;
    constexpr int SHARE_B = kThreads / BN > 0 ? kThreads / BN : 1;
    int32_t *sum_a = reinterpret_cast<int32_t *>(lds);        // [SHARE_A][BM]
    int32_t *sum_b = sum_a + SHARE_A * BM;                    // [SHARE_B][BN]
    {
        uint32_t wa = 0, wb = 0;
#pragma unroll
        for (int i = 0; i < P; ++i) wa += pop_a[i] << i;
#pragma unroll
        for (int i = 0; i < Q; ++i) wb += pop_b[i] << i;
        sum_a[(tid / BM) * BM + tid % BM] = (int32_t)wa;
        sum_b[(tid / BN) * BN + tid % BN] = (int32_t)wb;
    }
    __syncthreads();
    // C = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw, in wrapping 32-bit arithmetic (C itself fits)
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    const uint32_t base = (uint32_t)g.K * ca * cw;

    // Accumulator layout of the 32x32 MFMA: lane l, register v holds
    //   row = 8*(v/4) + 4*(l/32) + v%4, column = l%32.
    const int col = lane & 31, rsub = (lane >> 5) * 4;
    uint32_t col_term[WN];
    float sw[WN];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        const int nl = (wave_n * WN + bj) * 32 + col;
        uint32_t pw = 0;
#pragma unroll
        for (int h = 0; h < SHARE_B; ++h) pw += (uint32_t)sum_b[h * BN + nl];
        col_term[bj] = base - 2u * ca * pw;
        const int64_t n = n0 + nl;
        sw[bj] = (g.w_scale && n < g.N) ? half_bits_to_float(g.w_scale[n]) : 1.0f;
    }

    // The output mode and the border test are uniform over the workgroup: pick one of six
    // straight-line store sequences instead of testing per element.
    const int64_t m_lane = m0 + wave_m * WM * 32 + rsub;  // row of (bi = 0, v4 = 0, r = 0)
    const int64_t n_lane = n0 + wave_n * WN * 32 + col;   // column of bj = 0
    auto emit = [&](auto guard_c, auto i32_c, auto f16_c) __attribute__((always_inline)) {
        constexpr bool GUARD = decltype(guard_c)::value, I32 = decltype(i32_c)::value, F16 = decltype(f16_c)::value;
        int32_t *ci = I32 ? g.c_i32 + m_lane * g.N + n_lane : nullptr;
        uint16_t *ch = F16 ? g.c_f16 + m_lane * g.N + n_lane : nullptr;
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int ml = (wave_m * WM + bi) * 32 + 8 * v4 + rsub;  // first of four consecutive rows
                int4 pa = *reinterpret_cast<const int4 *>(sum_a + ml);
#pragma unroll
                for (int h = 1; h < SHARE_A; ++h) {
                    const int4 more = *reinterpret_cast<const int4 *>(sum_a + h * BM + ml);
                    pa.x += more.x; pa.y += more.y; pa.z += more.z; pa.w += more.w;
                }
                const uint32_t row_term[4] = {0u - 2u * cw * (uint32_t)pa.x, 0u - 2u * cw * (uint32_t)pa.y,
                                              0u - 2u * cw * (uint32_t)pa.z, 0u - 2u * cw * (uint32_t)pa.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int64_t row = (int64_t)(bi * 32 + 8 * v4 + r);  // relative to m_lane
                    if (GUARD && m_lane + row >= g.M) continue;
                    float sa = 1.0f;
                    if constexpr (F16) sa = g.a_scale ? half_bits_to_float(g.a_scale[m_lane + row]) : 1.0f;
#pragma unroll
                    for (int bj = 0; bj < WN; ++bj) {
                        if (GUARD && n_lane + bj * 32 >= g.N) continue;
                        const uint32_t c = ((uint32_t)acc[bi][bj][4 * v4 + r] << 2) + row_term[r] + col_term[bj];
                        if constexpr (I32) ci[row * g.N + bj * 32] = (int32_t)c;
                        if constexpr (F16) ch[row * g.N + bj * 32] = float_to_half_bits((float)(int32_t)c * sa * sw[bj]);
                    }
                }
            }
        }
    };
    using T = std::true_type;
    using F = std::false_type;
    const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N);
    const bool i32 = g.c_i32 != nullptr, f16 = g.c_f16 != nullptr;
    if (interior) {
        if (i32 && !f16) emit(F{}, T{}, F{});
        else if (!i32 && f16) emit(F{}, F{}, T{});
        else emit(F{}, T{}, T{});
    } else {
        if (i32 && !f16) emit(T{}, T{}, F{});
        else if (!i32 && f16) emit(T{}, F{}, T{});
        else emit(T{}, T{}, T{});
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

// Tile choice: the 256 x 256 tile has the lowest expansion and LDS cost per MFMA but needs
// enough tiles to occupy the 256 CUs; otherwise 128 x 128.
template <int P, int Q>
hipError_t launch_pq(const GemmArgs &g, hipStream_t stream)
{
    const int64_t big = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big >= 192) return launch_variant<P, Q, 4, 4>(g, stream);
    return launch_variant<P, Q, 2, 2>(g, stream);
}

// One translation unit per activation width instantiates launch_p<P>.
template <int P>
hipError_t launch_p(const GemmArgs &g, hipStream_t stream)
{
    switch (g.q) {
    case 1: return launch_pq<P, 1>(g, stream);
    case 2: return launch_pq<P, 2>(g, stream);
    case 3: return launch_pq<P, 3>(g, stream);
    case 4: return launch_pq<P, 4>(g, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace mfma
}  // namespace apmm
