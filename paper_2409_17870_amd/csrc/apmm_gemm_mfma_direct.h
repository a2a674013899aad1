// Design A without LDS: every wave expands its own MFMA operands in registers.
//
// Same algebra as apmm_gemm_mfma_impl.h (codes u on the matrix unit, C = 4S - 2cw PA - 2ca PW +
// K ca cw), different data movement.  On gfx950 a wave that owns its SIMD alone has about 17 issue
// cycles per 32-cycle MFMA for everything else; a ds_read_b128 costs ~20 and a ds_write_b128 ~40 of
// them, a VALU instruction 4.  Staging the expanded tiles through LDS (one expansion per workgroup,
// then 0.5 reads + 0.25 writes per MFMA) therefore costs more issue time than letting each of the
// two waves that share a fragment expand it again from the packed planes, which are 4-8x smaller
// than the operand bytes and come straight from L1/L2 into registers (paper Sec. 4.1: the planes are
// stored so that one 16-byte load per plane brings a row's 128 k).  There is no LDS traffic, no
// barrier in the k loop and nothing but C reaches global memory (paper Sec. 4.2).
//
// E2M1 (fp4) operands hold 2-bit codes.  q <= 2; p = 1, 2 or 4: 4-bit activation codes are split
// into two 2-bit plane groups, u = 4 u_hi + u_lo, and K is swept once per group with the MFMA's
// power-of-two operand scale set to 4 resp. 1, so that the one accumulator receives
// S = 4 sum u_hi uw + sum u_lo uw (the plane-group form of the paper's shift-and-add, done by the
// matrix unit's scale input).  Workgroup = 2 x 2 waves, wave tile (32*WM) x (32*WN).
// Stage = two packed k blocks = four MFMA k steps of 64.  Lane l of a wave owns, for each of its
// WM + WN row blocks, row l % 32 and k block l / 32 of the stage: per plane one 16-byte load = the
// four 32-k word groups gq = 0..3 of that row.  MFMA k step ks multiplies word group gq = ks of both
// lane halves; the lane's 32 codes of that group, expanded to nibbles, are exactly its 16 operand
// bytes.  The expansion of k step ks+1 (and, at the end of a stage, of step 0 of the next stage) is
// interleaved with the MFMAs of step ks, two output dwords per MFMA.  The raw words of the next
// stage are loaded at the start of the current one (double buffered in registers).
#pragma once
#include "apmm_mfma_common.h"

namespace apmm {
namespace mfma {

template <int P, int Q, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_mfma_direct_kernel(GemmArgs g, int tiles_n, int tiles_total)
{
    static_assert((P == 1 || P == 2 || P == 4) && Q <= 2, "E2M1 patterns are linear in the code only up to 3");
    constexpr bool FP4 = true;
    constexpr int GROUPS = P > 2 ? 2 : 1;    // 2-bit plane groups of the activations
    constexpr int PG = P / GROUPS;           // planes per group
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int KS = 4;                    // MFMA k steps per stage (= word groups of a k block)
    constexpr int PER_KS = WM * WN;          // MFMAs per k step
    constexpr int FRAGS = WM + WN;           // operand fragments per k step
    constexpr int TASKS = 4 * FRAGS;         // expansion dwords per k step
    static_assert(TASKS % PER_KS == 0, "expansion tasks must spread evenly over the MFMAs of a k step");
    constexpr int TPM = TASKS / PER_KS;      // tasks per MFMA
    typedef typename Acc<FP4>::type acc_t;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int r32 = lane & 31, kh = lane >> 5;
    const int lid = xcd_tile_id(blockIdx.x, tiles_total);
    const int tm = lid / tiles_n, tn = lid % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // per row block: address of (row, plane 0, words 0..3) in this lane's k block of stage 0
    const int64_t rows_a = round_up(g.M, kRowBlock), rows_b = round_up(g.N, kRowBlock);
    const uint4 *pa_src[WM], *pb_src[WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi) {
        int64_t row = m0 + (wave_m * WM + bi) * 32 + r32;
        if (row >= rows_a) row = rows_a - 1;  // rows past the operand: read a valid row, never stored
        pa_src[bi] = reinterpret_cast<const uint4 *>(g.a + tile_row_word(row, kh, g.nkb, P, 0));
    }
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        int64_t row = n0 + (wave_n * WN + bj) * 32 + r32;
        if (row >= rows_b) row = rows_b - 1;
        pb_src[bj] = reinterpret_cast<const uint4 *>(g.w + tile_row_word(row, kh, g.nkb, Q, 0));
    }
    constexpr int kPlaneVec = kPlaneWords / 4;             // uint4 between planes of a tile
    constexpr int kStageVecA = 2 * P * kPlaneVec, kStageVecB = 2 * Q * kPlaneVec;  // uint4 per stage (2 k blocks)

    uint4 ra[2][WM][PG], rb[2][WN][Q];  // raw plane words, double buffered by stage parity
    int grp = 0;                        // plane group being swept
    auto load_stage = [&](auto buf_c, int64_t st) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
#pragma unroll
        for (int bi = 0; bi < WM; ++bi)
#pragma unroll
            for (int i = 0; i < PG; ++i) ra[buf][bi][i] = pa_src[bi][st * kStageVecA + (grp * PG + i) * kPlaneVec];
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
#pragma unroll
            for (int i = 0; i < Q; ++i) rb[buf][bj][i] = pb_src[bj][st * kStageVecB + i * kPlaneVec];
    };

    acc_t acc[WM][WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi)
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0;

    v4i af[2][WM], bf[2][WN];
    // dword d of fragment f (f < WM: A block f, else B block f - WM) of k step ks, from buffer buf
    auto expand = [&](auto buf_c, auto ks_c, auto f_c, auto d_c) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value, f = decltype(f_c)::value,
                      d = decltype(d_c)::value;
        auto word = [](const uint4 &v) { return ks == 0 ? v.x : ks == 1 ? v.y : ks == 2 ? v.z : v.w; };
        if constexpr (f < WM) {
            uint32_t w[PG];
#pragma unroll
            for (int i = 0; i < PG; ++i) w[i] = word(ra[buf][f][i]);
            af[ks & 1][f][d] = GROUPS == 1 ? (int)expand_dword<PG, FP4>(w, d) : (int)expand_group_dword<PG>(w, d, grp * PG);
        } else {
            uint32_t w[Q];
#pragma unroll
            for (int i = 0; i < Q; ++i) w[i] = word(rb[buf][f - WM][i]);
            bf[ks & 1][f - WM][d] = (int)expand_dword<Q, FP4>(w, d);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    const int64_t nst = g.nkb / 2;  // the packed K is a multiple of 512: an even number of whole stages
    int scale_a = 127;

    // one stage with its raw words in buffer `buf`; loads stage st+1 (clamped) into the other buffer
    auto stage = [&](auto buf_c, int64_t st) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
        using Other = std::integral_constant<int, buf ^ 1>;
        load_stage(Other{}, st + 1 < nst ? st + 1 : st);  // the surplus load of the last stage is discarded
        __builtin_amdgcn_sched_barrier(0);
        static_for<KS * PER_KS>([&](auto i_c) __attribute__((always_inline)) {
            constexpr int i = decltype(i_c)::value;
            constexpr int ks = i / PER_KS, j = i % PER_KS, bi = j / WN, bj = j % WN;
            acc[bi][bj] = Acc<FP4>::mma_scaled(af[ks & 1][bi], bf[ks & 1][bj], acc[bi][bj], scale_a);
            // this MFMA's share of the next k step's operands (after the last step: step 0 of stage st+1)
            static_for<TPM>([&](auto t_c) __attribute__((always_inline)) {
                constexpr int task = j * TPM + decltype(t_c)::value;
                using F = std::integral_constant<int, task / 4>;
                using D = std::integral_constant<int, task % 4>;
                if constexpr (ks + 1 < KS)
                    expand(buf_c, std::integral_constant<int, ks + 1>{}, F{}, D{});
                else
                    expand(Other{}, I0{}, F{}, D{});
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (grp = 0; grp < GROUPS; ++grp) {
        scale_a = 127 + grp * PG;  // E8M0 exponent: the codes of this group weigh 2^(grp * PG)
        load_stage(I0{}, 0);
        // fragments of (stage 0, k step 0)
        static_for<FRAGS>([&](auto f_c) __attribute__((always_inline)) {
            static_for<4>([&](auto d_c) __attribute__((always_inline)) { expand(I0{}, I0{}, f_c, d_c); });
        });
        for (int64_t st = 0; st < nst; st += 2) {
            stage(I0{}, st);
            stage(I1{}, st + 1);
        }
    }

    // recovery terms: the code sums of the rows come with the packed operands
    const int rsub = kh * 4;
    const int64_t m_lane = m0 + wave_m * WM * 32 + rsub, n_lane = n0 + wave_n * WN * 32 + r32;
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

template <int P, int Q, int WM, int WN>
hipError_t launch_direct_variant(const GemmArgs &g, hipStream_t stream)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int64_t tiles = tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_mfma_direct_kernel<P, Q, WM, WN>), dim3((unsigned)tiles), dim3(256), 0, stream, g,
                       (int)tiles_n, (int)tiles);
    return hipGetLastError();
}

}  // namespace mfma
}  // namespace apmm
