// Design A for outputs too small to give every compute unit a large tile: the four waves of a workgroup split K.
//
// The algebra is that of apmm_gemm_mfma_direct.h (paper Sec. 3.2: the shift-and-add over plane pairs, moved in
// front of the multiplier; recovery terms as the accumulator's start value).  What differs is who shares what.
// There the four waves of a workgroup own four parts of the output tile and each sweeps all of K, so that two
// waves load (and expand) every packed fragment; the tiles that fit the register file then ask the L1 of a compute
// unit for more bytes per MFMA than it delivers, most of all with activations in the 6-bit field form, and a
// prefill of a few hundred tokens leaves a third of the chip without a tile.  Here every wave owns the WHOLE
// workgroup tile (WM x WN blocks of 32 x 32, as many as the accumulator registers hold) and a quarter of the
// stages of K (paper Sec. 4.2 item 2 partitions K in time; this partitions it across waves as well): no fragment
// is loaded twice inside a compute unit, the bytes per MFMA are those of the largest wave tile, and a 512 x 5120
// output is 256 tiles of 64 x 160 instead of 160 of 128 x 128.  The four partial tiles meet in LDS once, at the
// end: every wave writes the blocks it does not own, and after one barrier adds the three other partials of the
// blocks it owns (fp32 sums of integers below 2^24: exact in any order) and stores them.  The recovery terms
// start the accumulators of wave 0 only.
#pragma once
#include <hip/hip_ext.h>

#include "apmm_mfma_common.h"

namespace apmm {
namespace mfma {

// Owner (wave) of block (bi, bj) of the workgroup tile in the final reduction: every wave's blocks lie in one
// row block, so that it needs one set of token scales.
constexpr int ksplit_owner(int wm, int wn, int bi, int bj)
{
    return wm == 1 ? bj * 4 / wn : wm == 2 ? 2 * bi + (bj >= (wn + 1) / 2 ? 1 : 0) : bi;
}
constexpr int ksplit_lds_bytes(int wm, int wn) { return wm * wn * 3 * 4 * 64 * 16; }

template <int P, int Q, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_mfma_ksplit_kernel(const uint32_t *a_arg, const uint32_t *w_arg, int32_t *ci_arg,
                                                               uint16_t *cf_arg, int m_arg, int n_arg, int k_arg, int nkb_arg,
                                                               int tiles_n, int tiles_m_xn, const uint16_t *ws_arg,
                                                               const uint16_t *as_arg)
{
    static_assert(P >= 1 && P <= 4 && Q >= 1 && Q <= 4, "instantiated for codes of up to four bits");
    static_assert(WM == 1 || WM == 2 || WM == 4, "row blocks per tile");
    static_assert(WM * WN <= 13, "three partial copies of every block must fit the 160 KB of LDS");
    extern __shared__ __align__(16) float4 red[];  // [block][partial 0..2][register quad 0..3][lane]
    constexpr bool AF = activation_field_form(P);
    constexpr int SLOTS_A = activation_slots(P);
    constexpr int NB = WM * WN;
    constexpr int KS = 4;
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r32 = lane & 31, kh = lane >> 5;
    // Workgroups are dealt round-robin to the 8 XCDs, each with an L2 of its own.  The tile grid is cut into
    // 8 / xn x xn parts, one per XCD, and a part is walked down its columns: the workgroups that run together on an
    // XCD share the packed rows of a few column tiles and of the part's row tiles (tiles_m_xn = tiles_m | log2(xn) << 28).
    const int tiles_m = tiles_m_xn & 0x0fffffff, xn_log = tiles_m_xn >> 28;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int part_m = (tiles_m + (8 >> xn_log) - 1) >> (3 - xn_log), part_n = (tiles_n + (1 << xn_log) - 1) >> xn_log;
    const int tm = (xcd >> xn_log) * part_m + idx % part_m, tn = (xcd & ((1 << xn_log) - 1)) * part_n + idx / part_m;
    if (tm >= tiles_m || tn >= tiles_n) return;  // the grid is padded to 8 equal parts
    const int64_t M = m_arg, N = n_arg;
    const int64_t m0 = (int64_t)tm * (32 * WM), n0 = (int64_t)tn * (32 * WN);
    const int64_t nrb_a = (M + 31) / 32, nrb_b = (N + 31) / 32;
    const int32_t *a_sum = reinterpret_cast<const int32_t *>(a_arg + row_sum_word(nrb_a * 32, nkb_arg, SLOTS_A));
    const int32_t *w_sum = reinterpret_cast<const int32_t *>(w_arg + row_sum_word(nrb_b * 32, nkb_arg, Q));

    // this wave's stages of K: nst stages of two k blocks, dealt as evenly as they go
    const int nst = nkb_arg / 2;
    const int s_begin = wave * (nst / 4) + (wave < nst % 4 ? wave : nst % 4);
    const int s_count = nst / 4 + (wave < nst % 4 ? 1 : 0);
    const int s_end = s_begin + s_count;

    // Addresses: a uniform pointer per block (row blocks past the operand read the last one; never stored) plus
    // one lane offset per operand: row r32 of k block kh of a stage.
    constexpr int kSlotBytes = kPlaneWords * 4;
    constexpr int kStageBytesA = 2 * SLOTS_A * kSlotBytes, kStageBytesB = 2 * Q * kSlotBytes;
    const uint32_t voff_a = (uint32_t)(kh * SLOTS_A * kSlotBytes + r32 * 16);
    const uint32_t voff_b = (uint32_t)(kh * Q * kSlotBytes + r32 * 16);
    const char *pa_blk[WM], *pb_blk[WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi) {
        int64_t rb = m0 / 32 + bi;
        if (rb >= nrb_a) rb = nrb_a - 1;
        pa_blk[bi] = reinterpret_cast<const char *>(a_arg) + rb * nkb_arg * (int64_t)(SLOTS_A * kSlotBytes);
    }
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        int64_t rb = n0 / 32 + bj;
        if (rb >= nrb_b) rb = nrb_b - 1;
        pb_blk[bj] = reinterpret_cast<const char *>(w_arg) + rb * nkb_arg * (int64_t)(Q * kSlotBytes);
    }

    v16f acc[WM][WN];
    uint4 ra[2][WM][AF ? 6 : 2], rb[2][WN][2];  // raw words of a stage, by stage parity
    v4i af[2][AF ? 1 : WM], bf[2][WN];          // expanded fragments, by k step parity

    auto load_stage_of = [&](auto as_c, auto bs_c, auto buf_c, int st, int slot_a, int slot_b) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
        constexpr bool AS = decltype(as_c)::value, BS = decltype(bs_c)::value;
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
            const char *src = pa_blk[bi] + (int64_t)st * kStageBytesA + voff_a;
            if constexpr (AF) {
#pragma unroll
                for (int sl = 0; sl < 6; ++sl) ra[buf][bi][sl] = *reinterpret_cast<const uint4 *>(src + sl * kSlotBytes);
            } else {
                ra[buf][bi][0] = *reinterpret_cast<const uint4 *>(src + slot_a * kSlotBytes);
                if constexpr (!AS) ra[buf][bi][1] = *reinterpret_cast<const uint4 *>(src + (slot_a + 1) * kSlotBytes);
            }
        }
#pragma unroll
        for (int bj = 0; bj < WN; ++bj) {
            const char *src = pb_blk[bj] + (int64_t)st * kStageBytesB + voff_b;
            rb[buf][bj][0] = *reinterpret_cast<const uint4 *>(src + slot_b * kSlotBytes);
            if constexpr (!BS) rb[buf][bj][1] = *reinterpret_cast<const uint4 *>(src + (slot_b + 1) * kSlotBytes);
        }
    };

    // First requests: the wave's first stage of the first sweep, then the code sums (wave 0 seeds the
    // accumulators with the recovery terms, the others start at zero).
    constexpr bool AS0 = !AF && pair_groups(P) == 0, BS0 = pair_groups(Q) == 0;
    constexpr int SLOT_A0 = 0, SLOT_B0 = pair_groups(Q) > 0 ? 0 : Q - 1;
    if (s_count > 0)
        load_stage_of(std::integral_constant<bool, AS0>{}, std::integral_constant<bool, BS0>{}, I0{}, s_begin, SLOT_A0, SLOT_B0);
    {
        float a_init[WM], b_init[WN];
#pragma unroll
        for (int bj = 0; bj < WN; ++bj) {
            int64_t n = n0 + bj * 32 + r32;
            if (n >= nrb_b * 32) n = nrb_b * 32 - 1;
            const float ct = (float)(int32_t)((uint32_t)k_arg * ca * cw - 2u * ca * (uint32_t)w_sum[n]);
            b_init[bj] = wave != 0 ? 0.f : kh == 0 ? 1.0f : ct;
        }
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
            int64_t m = m0 + bi * 32 + r32;
            if (m >= nrb_a * 32) m = nrb_a * 32 - 1;
            const float rt = -(float)(2u * cw * (uint32_t)a_sum[m]);
            a_init[bi] = wave != 0 ? 0.f : kh == 0 ? rt : 1.0f;
        }
        v16f zero;
#pragma unroll
        for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
        for (int bi = 0; bi < WM; ++bi)
#pragma unroll
            for (int bj = 0; bj < WN; ++bj)
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_init[bi], b_init[bj], zero, 0, 0, 0);
    }

    // One sweep of this wave's stages for the activation group at slot slot_a and the weight group at slot slot_b
    // (AS / BS: the group is a single one); exp_a + exp_b - 254 = 4 + the bit positions of the two groups.
    auto sweep = [&](auto as_c, auto bs_c, int slot_a, int slot_b, int exp_a, int exp_b, auto preloaded_c) __attribute__((always_inline)) {
        constexpr bool AS = decltype(as_c)::value, BS = decltype(bs_c)::value, PRELOADED = decltype(preloaded_c)::value;
        constexpr int PER_KS = NB;
        constexpr int FRAG0 = AF ? WM : 0, FRAGS = WM + WN;
        constexpr int TASKS = 4 * (FRAGS - FRAG0);
        constexpr int TPM = (TASKS + PER_KS - 1) / PER_KS;
        auto expand = [&](auto buf_c, auto ks_c, auto f_c, auto d_c) __attribute__((always_inline)) {
            constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value, f = decltype(f_c)::value,
                          d = decltype(d_c)::value;
            if constexpr (f < WM) {
                if constexpr (AF) {
                } else if constexpr (AS) {
                    af[ks & 1][f][d] = (int)fp4_single_dword<ks, d>(ra[buf][f][0]);
                } else {
                    af[ks & 1][f][d] = (int)fp4_pair_dword<ks, d>(ra[buf][f][0], ra[buf][f][1]);
                }
            } else {
                if constexpr (BS) bf[ks & 1][f - WM][d] = (int)fp4_single_dword<ks, d>(rb[buf][f - WM][0]);
                else bf[ks & 1][f - WM][d] = (int)fp4_pair_dword<ks, d>(rb[buf][f - WM][0], rb[buf][f - WM][1]);
            }
        };
        auto stage = [&](auto buf_c, int st) __attribute__((always_inline)) {
            constexpr int buf = decltype(buf_c)::value;
            using Other = std::integral_constant<int, buf ^ 1>;
            load_stage_of(as_c, bs_c, Other{}, st + 1 < s_end ? st + 1 : st, slot_a, slot_b);  // the surplus load is discarded
            __builtin_amdgcn_sched_barrier(0);
            static_for<KS * PER_KS>([&](auto i_c) __attribute__((always_inline)) {
                constexpr int i = decltype(i_c)::value;
                constexpr int ks = i / PER_KS, j = i % PER_KS, bi = j / WN, bj = j % WN;
                const v4i b = bf[ks & 1][bj];
                const v8i b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
                if constexpr (AF) {
                    auto raw = [&](auto w_c) __attribute__((always_inline)) {
                        constexpr int w = 6 * ks + decltype(w_c)::value;
                        return (int)vec_word<w & 3>(ra[buf][bi][w >> 2]);
                    };
                    const v8i a8 = {raw(std::integral_constant<int, 0>{}), raw(std::integral_constant<int, 1>{}),
                                    raw(std::integral_constant<int, 2>{}), raw(std::integral_constant<int, 3>{}),
                                    raw(std::integral_constant<int, 4>{}), raw(std::integral_constant<int, 5>{}), 0, 0};
                    acc[bi][bj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        a8, b8, acc[bi][bj], 2, 4, 0, exp_a, 0, exp_b + (BS ? fp4_single_exponent(ks) : 0));
                } else {
                    const v4i a = af[ks & 1][bi];
                    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
                    acc[bi][bj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        a8, b8, acc[bi][bj], 4, 4, 0, exp_a + (AS ? fp4_single_exponent(ks) : 0), 0,
                        exp_b + (BS ? fp4_single_exponent(ks) : 0));
                }
                static_for<TPM>([&](auto t_c) __attribute__((always_inline)) {
                    constexpr int task = j * TPM + decltype(t_c)::value;
                    if constexpr (task < TASKS) {
                        using F = std::integral_constant<int, FRAG0 + task / 4>;
                        using D = std::integral_constant<int, task % 4>;
                        if constexpr (ks + 1 < KS)
                            expand(buf_c, std::integral_constant<int, ks + 1>{}, F{}, D{});
                        else
                            expand(Other{}, I0{}, F{}, D{});
                    }
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        if (s_count == 0) return;
        if constexpr (!PRELOADED) load_stage_of(as_c, bs_c, I0{}, s_begin, slot_a, slot_b);
        static_for<FRAGS - FRAG0>([&](auto f_c) __attribute__((always_inline)) {
            using F = std::integral_constant<int, FRAG0 + decltype(f_c)::value>;
            static_for<4>([&](auto d_c) __attribute__((always_inline)) { expand(I0{}, I0{}, F{}, d_c); });
        });
        int st = s_begin;
        for (; st + 1 < s_end; st += 2) {
            stage(I0{}, st);
            stage(I1{}, st + 1);
        }
        if (st < s_end) stage(I0{}, st);
    };

    using T = std::true_type;
    using F = std::false_type;
    if constexpr (AF) {
        // one sweep per weight group; (ua / 8)(uw / 2) 2^6 = 4 ua uw
        if constexpr (pair_groups(Q) > 0) {
            sweep(F{}, F{}, 0, 0, 130, 130, T{});
            for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(F{}, F{}, 0, 2 * hb, 130, 130 + 2 * hb, F{});
            if constexpr (has_single_group(Q)) sweep(F{}, T{}, 0, Q - 1, 130, 130 + Q - 1, F{});
        } else {
            sweep(F{}, T{}, 0, 0, 130, 130, T{});
        }
    } else if constexpr (pair_groups(P) > 0) {
        if constexpr (pair_groups(Q) > 0) {
            sweep(F{}, F{}, 0, 0, 129, 129, T{});
            for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(F{}, F{}, 0, 2 * hb, 129, 129 + 2 * hb, F{});
            if constexpr (has_single_group(Q)) sweep(F{}, T{}, 0, Q - 1, 129, 129 + Q - 1, F{});
        } else {
            sweep(F{}, T{}, 0, Q - 1, 129, 129 + Q - 1, T{});
        }
        for (int ha = 1; ha < pair_groups(P); ++ha) {
            for (int hb = 0; hb < pair_groups(Q); ++hb) sweep(F{}, F{}, 2 * ha, 2 * hb, 129 + 2 * ha, 129 + 2 * hb, F{});
            if constexpr (has_single_group(Q)) sweep(F{}, T{}, 2 * ha, Q - 1, 129 + 2 * ha, 129 + Q - 1, F{});
        }
        if constexpr (has_single_group(P)) {
            for (int hb = 0; hb < pair_groups(Q); ++hb) sweep(T{}, F{}, P - 1, 2 * hb, 129 + P - 1, 129 + 2 * hb, F{});
            if constexpr (has_single_group(Q)) sweep(T{}, T{}, P - 1, Q - 1, 129 + P - 1, 129 + Q - 1, F{});
        }
    } else {  // P == 1
        if constexpr (pair_groups(Q) > 0) {
            sweep(T{}, F{}, 0, 0, 129, 129, T{});
            for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(T{}, F{}, 0, 2 * hb, 129, 129 + 2 * hb, F{});
            if constexpr (has_single_group(Q)) sweep(T{}, T{}, 0, Q - 1, 129, 129 + Q - 1, F{});
        } else {
            sweep(T{}, T{}, 0, 0, 129, 129, T{});
        }
    }
    // ---- the four partial tiles meet ----
    // Scales of the blocks this wave will store, requested before the exchange so that they are there after it:
    // the 16 token scales of this lane's rows (all of a wave's blocks lie in row block bi_own), one channel scale
    // per block.
    const int bi_own = WM == 1 ? 0 : WM == 2 ? wave >> 1 : wave;
    const int64_t m_own = m0 + bi_own * 32 + 4 * kh;  // row of register v: m_own + 8 (v / 4) + v % 4
    // (Unconditional loads from clamped addresses, one uniform branch around each set: a load under a per-lane
    // condition is followed by a wait, and 26 such waits in a row cost 2 us here.)
    uint32_t sa_bits[16], sw_bits[NB];
#pragma unroll
    for (int v = 0; v < 16; ++v) sa_bits[v] = 0x3c00u;
#pragma unroll
    for (int b = 0; b < NB; ++b) sw_bits[b] = 0x3c00u;
    if (cf_arg && as_arg) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int64_t m = m_own + 8 * (v / 4) + (v % 4);
            if (m >= M) m = M - 1;
            sa_bits[v] = as_arg[m];
        }
    }
    if (cf_arg && ws_arg) {
#pragma unroll
        for (int bj = 0; bj < WN; ++bj) {
            int64_t n = n0 + bj * 32 + r32;
            if (n >= N) n = N - 1;
            const uint32_t h = ws_arg[n];
#pragma unroll
            for (int bi = 0; bi < WM; ++bi) sw_bits[bi * WN + bj] = h;
        }
    }
    static_for<NB>([&](auto b_c) __attribute__((always_inline)) {
        constexpr int b = decltype(b_c)::value, bi = b / WN, bj = b % WN;
        constexpr int own = ksplit_owner(WM, WN, bi, bj);
        if (wave != own) {
            const int part = ((wave - own + 4) & 3) - 1;
            float4 *dst = red + (b * 3 + part) * 256 + lane;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                dst[q4 * 64] = make_float4(acc[bi][bj][4 * q4], acc[bi][bj][4 * q4 + 1], acc[bi][bj][4 * q4 + 2],
                                           acc[bi][bj][4 * q4 + 3]);
        }
    });
    __syncthreads();

    // Store of one owned block.  GUARD: border tile, every element tested.  PAIR (interior, even N, 4-byte aligned
    // fp16 output): neighbouring lanes hold neighbouring columns; rows are taken in pairs, the even lane of a lane
    // pair collects both columns of the first row, the odd lane both columns of the second (one lane exchange),
    // and each stores one dword instead of two halves.  NT: streaming stores when only one output is written.
    const bool interior = (m0 + 32 * WM <= M) && (n0 + 32 * WN <= N);
    const bool pair_ok = (N & 1) == 0 && (reinterpret_cast<uintptr_t>(cf_arg) & 3u) == 0;
    const bool single = !(ci_arg && cf_arg);
    const bool odd = lane & 1;
    float sa_f[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) sa_f[v] = half_bits_to_float((uint16_t)use_here(sa_bits[v]));
    static_for<NB>([&](auto b_c) __attribute__((always_inline)) {
        constexpr int b = decltype(b_c)::value, bi = b / WN, bj = b % WN;
        constexpr int own = ksplit_owner(WM, WN, bi, bj);
        if (wave != own) return;
        // all twelve reads of the three other partials in flight before the first add
        float4 t[12];
#pragma unroll
        for (int i = 0; i < 12; ++i) t[i] = red[(b * 3 + i / 4) * 256 + (i % 4) * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);
        v16f c = acc[bi][bj];
#pragma unroll
        for (int i = 0; i < 12; ++i) {
            c[4 * (i % 4)] += t[i].x; c[4 * (i % 4) + 1] += t[i].y; c[4 * (i % 4) + 2] += t[i].z; c[4 * (i % 4) + 3] += t[i].w;
        }
        const int64_t n = n0 + bj * 32 + r32;
        auto emit = [&](auto guard_c, auto i32_c, auto f16_c, auto pair_c, auto nt_c) __attribute__((always_inline)) {
            constexpr bool GUARD = decltype(guard_c)::value, I32 = decltype(i32_c)::value, F16 = decltype(f16_c)::value,
                           PAIR = decltype(pair_c)::value, NT = decltype(nt_c)::value;
            const float sw = half_bits_to_float((uint16_t)use_here(sw_bits[b]));
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m_own + 8 * (v / 4) + (v % 4);
                if (GUARD && (m >= M || n >= N)) continue;
                if constexpr (I32) {
                    int32_t *dst = ci_arg + m * N + n;
                    if constexpr (NT) __builtin_nontemporal_store((int32_t)c[v], dst);
                    else *dst = (int32_t)c[v];
                }
                if constexpr (F16 && !PAIR) cf_arg[m * N + n] = float_to_half_bits(c[v] * sa_f[v] * sw);
                if constexpr (F16 && PAIR) {
                    if (v % 2 == 0) {
                        const uint32_t h0 = float_to_half_bits(c[v] * sa_f[v] * sw);
                        const uint32_t h1 = float_to_half_bits(c[(v + 1) & 15] * sa_f[(v + 1) & 15] * sw);
                        const uint32_t give = odd ? h0 : h1, keep = odd ? h1 : h0;
                        const uint32_t got = (uint32_t)__builtin_amdgcn_mov_dpp((int)give, 0xB1, 0xf, 0xf, true);
                        const uint32_t word = odd ? (got | (keep << 16)) : (keep | (got << 16));
                        // odd lanes write the row below at the column to the left
                        uint32_t *dst = reinterpret_cast<uint32_t *>(cf_arg + (m + (odd ? 1 : 0)) * N + n - (odd ? 1 : 0));
                        if constexpr (NT) __builtin_nontemporal_store(word, dst);
                        else *dst = word;
                    }
                }
            }
        };
        if (ci_arg) {
            if (interior && single) emit(F{}, T{}, F{}, F{}, T{});
            else if (interior) emit(F{}, T{}, F{}, F{}, F{});
            else emit(T{}, T{}, F{}, F{}, F{});
        }
        if (cf_arg) {
            if (interior && pair_ok && single) emit(F{}, F{}, T{}, T{}, T{});
            else if (interior && pair_ok) emit(F{}, F{}, T{}, T{}, F{});
            else if (interior) emit(F{}, F{}, T{}, F{}, F{});
            else emit(T{}, F{}, T{}, F{}, F{});
        }
    });
}

template <int P, int Q, int WM, int WN>
hipError_t launch_ksplit_variant(const GemmArgs &g, hipStream_t stream)
{
    constexpr int BM = 32 * WM, BN = 32 * WN;
    constexpr int lds = ksplit_lds_bytes(WM, WN);
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    if (tiles_m >= (1 << 28) || tiles_n >= (1 << 28) || g.K > 0x7fffffffLL) return hipErrorInvalidValue;
    // Parts of the tile grid per XCD: 8 / xn along M times xn along N, the cut that leaves an XCD the fewest packed
    // bytes to read (its row tiles of A plus its column tiles of W).
    int xn_log = 0;
    double best = 0;
    for (int l = 0; l <= 3; ++l) {
        const int64_t pm = (tiles_m + (8 >> l) - 1) / (8 >> l), pn = (tiles_n + (1 << l) - 1) / (1 << l);
        const double bytes = (double)pm * BM * activation_slots(P) + (double)pn * BN * Q;
        if (l == 0 || bytes < best) { best = bytes; xn_log = l; }
    }
    const int64_t part_m = (tiles_m + (8 >> xn_log) - 1) / (8 >> xn_log), part_n = (tiles_n + (1 << xn_log) - 1) / (1 << xn_log);
    const int64_t tiles = 8 * part_m * part_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const int tiles_m_xn = (int)tiles_m | (xn_log << 28);
    auto kernel = gemm_mfma_ksplit_kernel<P, Q, WM, WN>;
    static thread_local int prepared_device = -1;  // the LDS limit is a per-device attribute of the function
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (prepared_device != dev) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        prepared_device = dev;
    }
    const KernelTiming timing = take_kernel_timing();
    note_kernel("gemm_mfma_ksplit_kernel<%d,%d,%d,%d>", P, Q, WM, WN);
    if (timing.start || timing.stop)
        hipExtLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(256), lds, stream, timing.start, timing.stop, 0, g.a, g.w,
                              g.c_i32, g.c_f16, (int)g.M, (int)g.N, (int)g.K, (int)g.nkb, (int)tiles_n, tiles_m_xn, g.w_scale,
                              g.a_scale);
    else
        hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(256), lds, stream, g.a, g.w, g.c_i32, g.c_f16, (int)g.M,
                           (int)g.N, (int)g.K, (int)g.nkb, (int)tiles_n, tiles_m_xn, g.w_scale, g.a_scale);
    return hipGetLastError();
}

}  // namespace mfma
}  // namespace apmm
