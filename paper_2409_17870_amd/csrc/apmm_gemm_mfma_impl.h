// Design A: bit planes recombined into matrix-unit operands on chip, one MFMA pass.
//
// Paper Sec. 3.2 recovers C = sum_i sum_j 2^(i+j) * D_ij from p*q one-bit products.  The
// matrix unit of gfx950 multiplies small numbers, not single bits, so the shift-and-add is
// moved in front of the multiplier: while the tile is copied from registers to LDS, the planes
// of each operand are combined into the code u = sum_i b_i 2^i; by paper Eq. 1 the value is
// v = sum_i (2*b_i - 1) * 2^i = 2u - (2^n - 1).  ONE MFMA pass gives S = sum_k ua_k * uw_k, and
// with the row sums of the codes (weighted popcounts of the planes, taken by the same threads
// that expand them)
//   C = sum_k (2 ua_k - ca)(2 uw_k - cw),   ca = 2^p - 1, cw = 2^q - 1
//     = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw,
//   PA[m] = sum_i 2^i * popcount(plane i of row m)  (padded k positions included: they hold the
//   code ca resp. cw in both operands, which is why the true K appears in the constant),
// which equals sum_ij 2^(i+j) D_ij.  This is the recovery of paper Sec. 4.2 done entirely in
// registers/LDS (nothing but C reaches global memory), at the cost of one MFMA pass instead
// of p*q, and the expansion costs one AND(-OR) per plane plus one rotate per output dword.
//
// Two operand formats:
//   INT8: code u as a byte, v_mfma_i32_32x32x32_i8, int32 accumulate (p, q <= 4 instantiated).
//   FP4 : code u as the E2M1 pattern 00uu, whose value is u/2 (patterns 0..3 are 0, 0.5, 1, 1.5),
//         v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales, fp32 accumulate.  Every product is a
//         multiple of 1/4 below 2.25 and every partial sum is exactly representable (K < 2^20),
//         so 16 * acc = 4 S is exact whatever the summation order.  Twice the MFMA rate of int8;
//         needs p, q <= 2.
//
// Workgroup = 256 threads = 2 x 2 waves; wave tile (32*WM) x (32*WN), workgroup tile
// BM x BN = (64*WM) x (64*WN).  One pipeline stage = four MFMA k steps = 128 k (INT8, one packed
// k block) or 256 k (FP4, two packed k blocks), double buffered in LDS (paper Sec. 4.2, items 2
// and 3: K partition and ping-pong buffers).  Per stage:
//   global -> registers : packed plane words of the stage after next
//   registers -> LDS    : expand the next stage to operand bytes in MFMA order, into the idle buffer
//   LDS -> MFMA         : ds_read_b128 fragments of the current buffer, one k step ahead of their MFMAs
// The three activities sit in one basic block and are interleaved instruction by instruction
// (one MFMA, then its share of expansion VALU work and LDS traffic), because a wave owns its
// SIMD alone (512 registers) and nothing else would cover the matrix unit while the VALU expands.
//
// LDS layout of one operand and stage: [ks = 4][row block][half = 2][row = 32][16 bytes], i.e. the
// 1 KB fragment of one MFMA (32 rows x one k step) is contiguous and lane l reads bytes
// 16*l .. 16*l+15: conflict free for ds_read_b128 and for the ds_write_b128 of the expansion.
// The k order inside a fragment is whatever the expansion produces; both operands use the same
// order, which is all the contraction needs.
#pragma once
#include "apmm_mfma_common.h"

namespace apmm {
namespace mfma {

constexpr int kStageSteps = 4;  // MFMA k steps per pipeline stage

// Per-thread share of one operand's workgroup tile and stage: UNITS units, one unit = (row, 32-k word
// group).  A stage spans SB packed k blocks (1 for INT8, 2 for FP4), i.e. 4*SB word groups per row.
template <int NB, int BX, int THREADS, bool FP4>
struct Loader {
    static constexpr int SB = FP4 ? 2 : 1;          // packed k blocks per stage
    static constexpr int R = THREADS / BX;          // threads sharing a row (BX = rows of the workgroup tile)
    static_assert(R == 1 || R == 2 || R == 4, "a row of the workgroup tile is shared by 1, 2 or 4 threads");
    static constexpr int UPB = kWordsPerRow / R;    // consecutive word groups a thread owns per k block
    static constexpr int UNITS = UPB * SB;          // units per thread and stage
    static constexpr int TPU = FP4 ? 4 : 8;         // output dwords (tasks) per unit
    static constexpr int TASKS = UNITS * TPU;       // expansion tasks per thread and stage
    uint32_t regs[UNITS][NB];
    uint32_t keep[SB];           // all ones, or zero for a k block past the end of K (FP4 stages only)
    const uint32_t *src0;        // word address of (row, plane 0, word gq0 * UPB) in k block 0, gq0 = tid / BX
    int lds_off[UNITS];          // byte offset of the unit's first 16-byte chunk inside the operand's stage

    // Unit s of a thread: k block s / UPB of the stage, word group gq0 * UPB + s % UPB of that block,
    // so that a thread's words of one plane and k block are consecutive (one 4-, 8- or 16-byte load).
    __device__ __forceinline__ void init(const uint32_t *packed, int64_t row0, int64_t rows_p, int64_t nkb,
                                         int tid)
    {
        const int row = tid % BX, gq0 = tid / BX;
        int64_t grow = row0 + row;
        if (grow >= rows_p) grow = rows_p - 1;  // rows past the operand: read a valid row, never stored
        src0 = packed + tile_row_word(grow, 0, nkb, NB, 0) + gq0 * UPB;
#pragma unroll
        for (int s = 0; s < UNITS; ++s) {
            const int gqs = (s / UPB) * kWordsPerRow + gq0 * UPB + s % UPB;  // word group inside the stage
            // INT8: k step = word group, two 16-byte chunks (halves) per unit.
            // FP4 : k step = pair of word groups, the unit is one half.
            const int ks = FP4 ? gqs / 2 : gqs, half = FP4 ? gqs % 2 : 0;
            lds_off[s] = ((ks * (BX / 32) + row / 32) * 2 + half) * 512 + (row % 32) * 16;
        }
#pragma unroll
        for (int b = 0; b < SB; ++b) keep[b] = 0xffffffffu;
    }
    // Stage st covers k blocks st*SB .. st*SB+SB-1.  A block past the end is read from the last
    // block and flagged; mask() later turns it into all-zero planes (code 0 in both operands adds
    // nothing to S, PA or PW).  The flag is applied a stage later so that the loads stay in flight.
    __device__ __forceinline__ void fetch(int64_t st, int64_t nkb)
    {
#pragma unroll
        for (int b = 0; b < SB; ++b) {
            int64_t kb = st * SB + b;
            keep[b] = 0xffffffffu;
            if (SB > 1 && kb >= nkb) {
                kb = nkb - 1;
                keep[b] = 0u;
            }
            const uint32_t *blk = src0 + kb * (kPlaneWords * NB);
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int u = 0; u < UPB; ++u) regs[b * UPB + u][i] = blk[i * kPlaneWords + u];
        }
    }
    __device__ __forceinline__ void mask()
    {
        if (SB == 1) return;
#pragma unroll
        for (int s = 0; s < UNITS; ++s)
#pragma unroll
            for (int i = 0; i < NB; ++i) regs[s][i] &= keep[s / UPB];
    }
    // whole share at once (prologue)
    __device__ __forceinline__ void expand_to_lds(uint8_t *stage) const
    {
        uint32_t o[4];
#pragma unroll
        for (int task = 0; task < TASKS; ++task) expand_task(stage, task, o);
    }
    // one output dword of the share: task = TPU * unit + t; every fourth task stores 16 bytes to LDS
    __device__ __forceinline__ void expand_task(uint8_t *stage, int task, uint32_t (&o)[4]) const
    {
        const int s = task / TPU, t = task % TPU;
        o[t % 4] = expand_dword<NB, FP4>(regs[s], t);
        if (t % 4 == 3)
            *reinterpret_cast<uint4 *>(stage + lds_off[s] + (t / 4) * 512) = make_uint4(o[0], o[1], o[2], o[3]);
    }
};

// Tile shape: GM x GN waves, each owning WM x WN blocks of 32 x 32.
template <int P, int Q, int WM, int WN, int GM, int GN, bool FP4>
__global__ __launch_bounds__(64 * GM * GN) void gemm_mfma_kernel(GemmArgs g, int tiles_n, int tiles_total)
{
    static_assert(!FP4 || (P <= 2 && Q <= 2), "E2M1 patterns are linear in the code only up to 3");
    constexpr int kThreads = 64 * GM * GN;
    constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN;
    constexpr int KS = kStageSteps;
    constexpr int A_STAGE = BM * 32 * KS, B_STAGE = BN * 32 * KS;  // bytes: 1 KB per 32 rows and k step
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int SB = FP4 ? 2 : 1;
    extern __shared__ __align__(16) uint8_t lds[];
    typedef typename Acc<FP4>::type acc_t;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / GN, wave_n = wave % GN;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
    // tiles so that the packed rows it re-reads stay in its own L2.
    int lid = blockIdx.x;
    if ((tiles_total & 7) == 0) lid = (blockIdx.x & 7) * (tiles_total >> 3) + (blockIdx.x >> 3);
    const int tm = lid / tiles_n, tn = lid % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    typedef Loader<P, BM, kThreads, FP4> LoaderA;
    typedef Loader<Q, BN, kThreads, FP4> LoaderB;
    LoaderA la;
    LoaderB lb;
    la.init(g.a, m0, round_up(g.M, kRowBlock), g.nkb, tid);
    lb.init(g.w, n0, round_up(g.N, kRowBlock), g.nkb, tid);

    acc_t acc[WM][WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi)
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0;

    const int64_t nst = (g.nkb + SB - 1) / SB;  // pipeline stages
    const int64_t last = nst - 1;
    la.fetch(0, g.nkb);
    lb.fetch(0, g.nkb);
    la.mask();
    lb.mask();
    la.expand_to_lds(lds);
    lb.expand_to_lds(lds + A_STAGE);
    la.fetch(last < 1 ? last : 1, g.nkb);
    lb.fetch(last < 1 ? last : 1, g.nkb);
    __syncthreads();

    const int frag_a = (wave_m * WM) * 1024 + lane * 16;
    const int frag_b = A_STAGE + (wave_n * WN) * 1024 + lane * 16;

    constexpr int MFMAS = WM * WN * KS;              // MFMAs per stage and wave
    constexpr int PER_KS = WM * WN;                  // MFMAs per k step
    constexpr int READS = WM + WN;                   // fragment reads per k step
    constexpr int TASKS_A = LoaderA::TASKS, TASKS = LoaderA::TASKS + LoaderB::TASKS;  // expansion dwords per thread and stage

    for (int64_t st = 0; st < nst; ++st) {
        const uint8_t *cur = lds + (st & 1) * STAGE;
        uint8_t *nxt = lds + ((st + 1) & 1) * STAGE;

        // raw planes of stage st+1 are in registers; start the loads of st+2 right away
        LoaderA ea = la;
        LoaderB eb = lb;
        ea.mask();
        eb.mask();
        const int64_t sf = (st + 2 <= last) ? st + 2 : last;  // clamped: the surplus fetches are discarded
        la.fetch(sf, g.nkb);
        lb.fetch(sf, g.nkb);
        v4i af[2][WM], bf[2][WN];
        // fragment r of k step ks: r = 0 -> A block 0, r = 1..WN -> B blocks, then the other A blocks
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
            // prefetch the fragments of the next k step, spread over this step's MFMAs
            if constexpr (ks + 1 < KS) {
                static_for<READS>([&](auto r_c) __attribute__((always_inline)) {
                    if constexpr (decltype(r_c)::value * PER_KS / READS == j)
                        read_frag(std::integral_constant<int, ks + 1>{}, r_c);
                });
            }
            acc[bi][bj] = Acc<FP4>::mma(af[ks & 1][bi], bf[ks & 1][bj], acc[bi][bj]);
            // this MFMA's share of the expansion of stage st+1 into the idle buffer (in the last
            // iteration it rewrites the stage already there: harmless, and keeps the body branch free)
            static_for<TASKS>([&](auto t_c) __attribute__((always_inline)) {
                constexpr int task = decltype(t_c)::value;
                if constexpr (task * MFMAS / TASKS == i) {
                    if constexpr (task < TASKS_A)
                        ea.expand_task(nxt, task, oa);
                    else
                        eb.expand_task(nxt + A_STAGE, task - TASKS_A, ob);
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();
    }

    // recovery terms: the code sums of the rows come with the packed operands
    const int col = lane & 31, rsub = (lane >> 5) * 4;
    const int64_t rows_a = round_up(g.M, kRowBlock), rows_b = round_up(g.N, kRowBlock);
    const int64_t m_lane = m0 + wave_m * WM * 32 + rsub, n_lane = n0 + wave_n * WN * 32 + col;
    const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N);
    uint32_t pw[WN];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        const int64_t n = n_lane + bj * 32;
        pw[bj] = (uint32_t)g.w_sum[n < rows_b ? n : rows_b - 1];
    }
    store_wave_tile<P, Q, WM, WN, FP4>(
        g, acc, m_lane, n_lane, interior,
        [&](int bi, int v4) {
            int64_t m = m_lane + bi * 32 + 8 * v4;  // four consecutive rows, 16-byte aligned
            if (m + 4 > rows_a) m = rows_a - 4;     // past the operand: any valid address, never stored
            return *reinterpret_cast<const int4 *>(g.a_sum + m);
        },
        pw);
}

template <int P, int Q, int WM, int WN, int GM, int GN, bool FP4>
hipError_t launch_variant(const GemmArgs &g, hipStream_t stream)
{
    constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN, threads = 64 * GM * GN;
    constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * 32 * kStageSteps;
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int64_t tiles = tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kernel = gemm_mfma_kernel<P, Q, WM, WN, GM, GN, FP4>;
    static bool attr_set = false;  // raising the dynamic LDS limit is idempotent; a race here is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(threads), lds_bytes, stream, g, (int)tiles_n,
                       (int)tiles);
    return hipGetLastError();
}

// Tile choice.  The 256 x 256 tile has the lowest expansion and LDS cost per MFMA but the grid must
// also fill the 256 CUs: estimate each candidate as (rounds of 256 tiles) x (tile area) x (relative
// cost per MFMA of that tile shape, measured) and take the cheapest.
template <int P, int Q, bool FP4>
hipError_t launch_tiles(const GemmArgs &g, hipStream_t stream)
{
    struct Cand { int bm, bn; double cost; };
    // measured on MI355X, per unit of tile area relative to 256 x 256: the smaller tiles expand more
    // operand bytes per MFMA, which costs more where the VALU is the limit (int8 with 4-bit planes)
    const Cand cands[4] = {{256, 256, 1.0}, {256, 128, FP4 ? 1.2 : 1.55}, {128, 256, FP4 ? 1.2 : 1.45},
                           {128, 128, FP4 ? 1.2 : 1.55}};
    int best = 0;
    double best_t = 0;
    // debugging aid: APMM_MFMA_TILE=0..3 forces a candidate
    static const char *forced = std::getenv("APMM_MFMA_TILE");
    if (forced && forced[0] >= '0' && forced[0] <= '3') {
        best = forced[0] - '0';
    } else
    for (int c = 0; c < 4; ++c) {
        const int64_t tiles = ((g.M + cands[c].bm - 1) / cands[c].bm) * ((g.N + cands[c].bn - 1) / cands[c].bn);
        const double t = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn * cands[c].cost;
        if (c == 0 || t < best_t) {
            best = c;
            best_t = t;
        }
    }
    switch (best) {
    case 0: return launch_variant<P, Q, 4, 4, 2, 2, FP4>(g, stream);
    case 1: return launch_variant<P, Q, 4, 2, 2, 2, FP4>(g, stream);
    case 2: return launch_variant<P, Q, 2, 4, 2, 2, FP4>(g, stream);
    default: return launch_variant<P, Q, 2, 2, 2, 2, FP4>(g, stream);
    }
}

// INT8 operands, one translation unit per activation width.
template <int P>
hipError_t launch_int8_p(const GemmArgs &g, hipStream_t stream)
{
    switch (g.q) {
    case 1: return launch_tiles<P, 1, false>(g, stream);
    case 2: return launch_tiles<P, 2, false>(g, stream);
    case 3: return launch_tiles<P, 3, false>(g, stream);
    case 4: return launch_tiles<P, 4, false>(g, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace mfma
}  // namespace apmm
