// Design A: bit planes recombined into matrix-unit operands in registers, E2M1 (fp4) MFMA.
//
// Paper Sec. 3.2 recovers C = sum_i sum_j 2^(i+j) * D_ij from p*q one-bit products.  The matrix unit of
// gfx950 multiplies small numbers, not single bits, so the shift-and-add is moved in front of the
// multiplier.  With the code u = sum_i b_i 2^i of an element, whose value is 2u - (2^n - 1) (paper Eq. 1),
//   C = sum_k (2 ua_k - ca)(2 uw_k - cw),   ca = 2^p - 1, cw = 2^q - 1
//     = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw,     S = sum_k ua_k uw_k,
//   PA[m], PW[n] = sums of the codes of a row over the padded K (they come with the packed operands;
//   padded k positions hold the code ca resp. cw in both operands, which is why the true K appears),
// which equals sum_ij 2^(i+j) D_ij.  The codes are cut into plane groups of two bits (and one of a single
// bit when the width is odd): u = sum_h 4^h u_h.  A 2-bit code is the E2M1 pattern 00uu = u/2, exactly, and
// S = sum_{h,h'} 4^(h+h') sum_k ua_h uw_h': K is swept once per pair of groups, every sweep adds into the
// SAME fp32 accumulator, and the factor 4^(h+h') (times 16 for the two halvings and the leading 4) is the
// MFMA's power-of-two operand scale: the paper's shift-and-add, done by the matrix unit.  The accumulator
// starts at -2 cw PA[m] - 2 ca PW[n] + K ca cw, so that it ends at C: every term is an integer and every
// partial sum stays below 2^24 (checked on the host), hence exact in any order.  Nothing but C reaches
// global memory (paper Sec. 4.2).
//
// Activations of 3 or 4 bits arrive in the field form (apmm_layout.h): their packed words ARE the E2M3 (fp6)
// operand, a 4-bit code u being the number u / 8, and the matrix unit multiplies fp6 by fp4 at the fp4 rate.
// They need no expansion and no sweep per activation group: K is swept once per weight group.
//
// Data movement: no LDS.  On gfx950 a wave that owns its SIMD alone has about 17 issue cycles per
// 32-cycle MFMA for everything else; a ds_read_b128 costs ~20 and a ds_write_b128 ~40 of them, a VALU
// instruction 4.  Staging expanded tiles through LDS therefore costs more issue time than letting each of
// the two waves that share a fragment expand it again from the packed words, which are 2-4x smaller than
// the operand bytes and come straight from L1/L2 into registers (paper Sec. 4.1: the planes are stored so
// that one 16-byte load brings a row's share of a k block).  There is no barrier in the k loop.
//
// Workgroup = 2 x 2 waves (4 x 1 for WM = 1), wave tile (32*WM) x (32*WN).  Stage = two packed k blocks = four MFMA k steps
// of 64.  Lane l of a wave owns, for each of its row blocks, row l % 32 and k block l / 32 of the stage:
// per group one or two 16-byte loads.  The expansion of k step ks+1 (and, at the end of a stage, of step 0
// of the next stage) is interleaved with the MFMAs of step ks; the raw words of the next stage are loaded
// at the start of the current one (double buffered in registers).
#pragma once
#include <hip/hip_ext.h>

#include "apmm_mfma_common.h"

namespace apmm {
namespace mfma {

// SPLIT = 1: the wave tile is computed in one go and stored at the end.
// SPLIT = 2: the wave tile is computed as two halves of WM / 2 row blocks, one after the other (each a full
// sweep of K), and the int32 stores of the first half are interleaved with the MFMAs of the second half's
// first stages, one element every other MFMA, so that half of the C traffic (which otherwise keeps the
// matrix unit idle for 6 - 7 us at 4096^2 outputs) runs under the k loop.  The price is less reuse per
// expanded fragment.
// SPLIT = 3: the same with an uneven cut, WM - 1 row blocks first and one row block second: three quarters of
// the output go out under the k loop (one element per MFMA of the second phase), the first phase keeps nearly
// the operand reuse of the whole tile, and only the short second phase pays for the stores and the low reuse.
// Both are used for interior tiles with int32 output only and K long enough to carry the stores.
// Arrangement of the four waves of a workgroup: 2 x 2, or 4 x 1 for wave tiles of a single row block (each row
// block of the workgroup tile is then loaded by one wave only, which matters when the activation operand is the
// heavy one: the 6-bit field form).
constexpr int waves_m(int wm) { return wm == 1 ? 4 : 2; }
constexpr int waves_n(int wm) { return 4 / waves_m(wm); }
constexpr int split_phases(int split) { return split == 1 ? 1 : 2; }
constexpr int split_rows(int wm, int split, int ph) { return split == 1 ? wm : split == 2 ? wm / 2 : (ph == 0 ? wm - 1 : 1); }
constexpr int split_row0(int wm, int split, int ph) { return ph == 0 ? 0 : split_rows(wm, split, 0); }
constexpr int split_store_every(int split) { return split == 3 ? 1 : 2; }  // MFMAs per stored element
// stages of phase 1 that carry the stores of phase 0 (KS = 4 k steps per stage)
constexpr int split_store_stages(int wm, int wn, int split)
{
    return split == 1 ? 0 : split_rows(wm, split, 0) * wn * 16 / (4 * split_rows(wm, split, 1) * wn / split_store_every(split));
}

// The arguments are plain scalars and pointers, the ones the first addresses depend on first: this file is built
// with kernel-argument preloading, so the first 14 dwords are in scalar registers when a wave starts and the
// prologue's first loads go out without a round trip to memory for the arguments.
template <int P, int Q, int WM, int WN, int SPLIT>
__global__ __launch_bounds__(256) void gemm_mfma_direct_kernel(const uint32_t *a_arg, const uint32_t *w_arg, int32_t *ci_arg,
                                                               uint16_t *cf_arg, int m_arg, int n_arg, int k_arg, int nkb_arg,
                                                               int tiles_n, int tiles_total, const uint16_t *ws_arg,
                                                               const uint16_t *as_arg)
{
    GemmArgs g;
    g.M = m_arg; g.N = n_arg; g.K = k_arg; g.nkb = nkb_arg;
    g.p = P; g.q = Q;
    g.a = a_arg; g.a_codes = nullptr; g.w = w_arg;
    g.a_sum = reinterpret_cast<const int32_t *>(a_arg + row_sum_word(round_up(m_arg, kRowBlock), nkb_arg, activation_slots(P)));
    g.w_sum = reinterpret_cast<const int32_t *>(w_arg + row_sum_word(round_up(n_arg, kRowBlock), nkb_arg, Q));
    g.c_i32 = ci_arg; g.c_f16 = cf_arg; g.w_scale = ws_arg; g.a_scale = as_arg;
    static_assert(P >= 1 && P <= 4 && Q >= 1 && Q <= 4, "instantiated for codes of up to four bits");
    static_assert(SPLIT >= 1 && SPLIT <= 3, "one phase, two even phases, or two uneven phases");
    static_assert(SPLIT == 1 || WM % 2 == 0, "the row blocks of a wave are cut in two");
    constexpr bool AF = activation_field_form(P);  // activations are ready-made fp6 operands
    constexpr int SLOTS_A = activation_slots(P);
    constexpr int PHASES = split_phases(SPLIT);
    constexpr int WMX = split_rows(WM, SPLIT, 0);  // row blocks of the largest phase (the first)
    constexpr int BM = 32 * WM * waves_m(WM), BN = 32 * WN * waves_n(WM);
    constexpr int KS = 4;                    // MFMA k steps per stage
    constexpr int STORE_EVERY = split_store_every(SPLIT);
    constexpr int STORE_STAGES = split_store_stages(WM, WN, SPLIT);  // stages of phase 1 that carry stores
    static_assert(STORE_STAGES % 2 == 0, "store schedule");
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    using I1 = std::integral_constant<int, 1>;
    using NoStore = std::integral_constant<int, -1>;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / waves_n(WM), wave_n = wave % waves_n(WM);
    const int r32 = lane & 31, kh = lane >> 5;
    const int lid = xcd_tile_id(blockIdx.x, tiles_total);
    const int tm = lid / tiles_n, tn = lid % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // per row block: address of (row, slot 0) in this lane's k block of stage 0
    const int64_t rows_a = round_up(g.M, kRowBlock), rows_b = round_up(g.N, kRowBlock);
    const uint4 *pa_src[WM], *pb_src[WN];
#pragma unroll
    for (int bi = 0; bi < WM; ++bi) {
        int64_t row = m0 + (wave_m * WM + bi) * 32 + r32;
        if (row >= rows_a) row = rows_a - 1;  // rows past the operand: read a valid row, never stored
        pa_src[bi] = reinterpret_cast<const uint4 *>(g.a + tile_row_word(row, kh, g.nkb, SLOTS_A, 0));
    }
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        int64_t row = n0 + (wave_n * WN + bj) * 32 + r32;
        if (row >= rows_b) row = rows_b - 1;
        pb_src[bj] = reinterpret_cast<const uint4 *>(g.w + tile_row_word(row, kh, g.nkb, Q, 0));
    }
    constexpr int kSlotVec = kPlaneWords / 4;                                    // uint4 between slots of a tile
    constexpr int kStageVecA = 2 * SLOTS_A * kSlotVec, kStageVecB = 2 * Q * kSlotVec;  // uint4 per stage (2 k blocks)

    // Accumulator layout of the 32x32 MFMA: lane l, register v holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    const int64_t m_lane = m0 + wave_m * WM * 32 + kh * 4, n_lane = n0 + wave_n * WN * 32 + r32;

    v16f acc[WM][WN];  // by row block of the wave tile; phase ph owns blocks split_row0(ph) ...
    uint4 ra[2][WMX][AF ? 6 : 2], rb[2][WN][2];  // raw words of a group (a single group uses [0] only; the field
                                                 // form all six slots), by stage parity
    v4i af[2][WMX], bf[2][WN];          // expanded fragments, by k step parity
    const int64_t nst = g.nkb / 2;      // the packed K is a multiple of 512: an even number of whole stages
    using I0 = std::integral_constant<int, 0>;

    // raw words of stage st of phase ph into buffer buf: the activation group at slot slot_a, the weight group at
    // slot slot_b (AS / BS: the group is a single one)
    auto load_stage_of = [&](auto ph_c, auto as_c, auto bs_c, auto buf_c, int64_t st, int slot_a, int slot_b)
                             __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_c)::value, buf = decltype(buf_c)::value;
        constexpr bool AS = decltype(as_c)::value, BS = decltype(bs_c)::value;
        constexpr int WMP = split_rows(WM, SPLIT, ph), ROW0 = split_row0(WM, SPLIT, ph);
#pragma unroll
        for (int bi = 0; bi < WMP; ++bi) {
            const uint4 *src = pa_src[ROW0 + bi];
            if constexpr (AF) {
#pragma unroll
                for (int sl = 0; sl < 6; ++sl) ra[buf][bi][sl] = src[st * kStageVecA + sl * kSlotVec];
            } else {
                ra[buf][bi][0] = src[st * kStageVecA + slot_a * kSlotVec];
                if constexpr (!AS) ra[buf][bi][1] = src[st * kStageVecA + (slot_a + 1) * kSlotVec];
            }
        }
#pragma unroll
        for (int bj = 0; bj < WN; ++bj) {
            rb[buf][bj][0] = pb_src[bj][st * kStageVecB + slot_b * kSlotVec];
            if constexpr (!BS) rb[buf][bj][1] = pb_src[bj][st * kStageVecB + (slot_b + 1) * kSlotVec];
        }
    };

    // Order of the first requests.  A kernel starts with cold caches and every dependent round trip to memory
    // costs about a microsecond, so everything the prologue needs is requested before anything is used: the
    // operands of stage 0 of the first sweep (slots 0 of both operands), then the code sums, then the scales.
    // (The one-phase 256 x 256 kernel has no registers to hold the operands while all 256 accumulators are being
    // set up; it requests them after that, one round trip later.  The kernels with 4-bit activations in the
    // field form measured 1 - 2 us slower with the early request and keep the old order too.)
    constexpr bool AS0 = !AF && pair_groups(P) == 0, BS0 = pair_groups(Q) == 0;  // the first sweep's groups
    constexpr bool PRELOAD = !(WM == 4 && WN == 4 && SPLIT == 1) && !AF;
    if constexpr (PRELOAD)
        load_stage_of(I0{}, std::integral_constant<bool, AS0>{}, std::integral_constant<bool, BS0>{}, I0{}, 0, 0, 0);
    uint32_t pw_raw[WN], pa_raw[WM];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        int64_t n = n_lane + bj * 32;
        if (n >= rows_b) n = rows_b - 1;
        pw_raw[bj] = (uint32_t)g.w_sum[n];
    }
    if constexpr (PRELOAD) {
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
            int64_t m = m0 + (wave_m * WM + bi) * 32 + r32;
            if (m >= rows_a) m = rows_a - 1;
            pa_raw[bi] = (uint32_t)g.a_sum[m];
        }
    }
    // Scales of the fp16 epilogue, requested now so that their latency is gone by the time they are needed:
    // sw[bj] for this lane's columns; the token scales of the wave's 32 * WM rows one row per lane (row
    // lane + 64 i in sa_rows[i]), handed to the lanes that need them by a lane permute in the epilogue.
    uint32_t sw_h[WN], sa_h[(WM + 1) / 2];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) sw_h[bj] = 0x3c00u;  // 1.0
#pragma unroll
    for (int i = 0; i < (WM + 1) / 2; ++i) sa_h[i] = 0x3c00u;
    if (PRELOAD && g.c_f16) {
#pragma unroll
        for (int bj = 0; bj < WN; ++bj) {
            const int64_t n = n_lane + bj * 32;
            if (g.w_scale && n < g.N) sw_h[bj] = g.w_scale[n];
        }
#pragma unroll
        for (int i = 0; i < (WM + 1) / 2; ++i) {
            const int64_t m = m0 + wave_m * WM * 32 + lane + 64 * i;
            if (g.a_scale && m < g.M && lane + 64 * i < 32 * WM) sa_h[i] = g.a_scale[m];
        }
    }

    // -- first uses from here on --
    // The accumulators start at the recovery terms rt[m] + ct[n], rt = -2 cw PA, ct = K ca cw - 2 ca PW: a
    // rank-2 matrix, written by one fp32 MFMA with k = 2 per block: A = (rt[m], 1), B = (1, ct[n]).
    // Lane l supplies row resp. column l % 32 of k index l / 32.  All values are integers below 2^24.
    float b_init[WN], a_init[WM];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        const float ct = (float)(int32_t)((uint32_t)g.K * ca * cw - 2u * ca * pw_raw[bj]);
        b_init[bj] = kh == 0 ? 1.0f : ct;
    }
    if constexpr (PRELOAD) {
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
            const float rt = -(float)(2u * cw * pa_raw[bi]);
            a_init[bi] = kh == 0 ? rt : 1.0f;
        }
    }
    // (the scales are kept as binary16 pairs through the k loop: registers are scarce there)
    uint32_t sw_raw[(WN + 1) / 2], sa_raw[(WM + 3) / 4];
    if constexpr (PRELOAD) {
#pragma unroll
        for (int i = 0; i < (WN + 1) / 2; ++i) sw_raw[i] = sw_h[2 * i] | ((2 * i + 1 < WN ? sw_h[2 * i + 1] : 0x3c00u) << 16);
#pragma unroll
        for (int i = 0; i < (WM + 3) / 4; ++i)
            sa_raw[i] = sa_h[2 * i] | ((2 * i + 1 < (WM + 1) / 2 ? sa_h[2 * i + 1] : 0x3c00u) << 16);
    } else {  // loaded and packed one by one (this form is the one the register allocator gets through without spilling)
#pragma unroll
        for (int i = 0; i < (WN + 1) / 2; ++i) sw_raw[i] = 0x3c003c00u;
#pragma unroll
        for (int i = 0; i < (WM + 3) / 4; ++i) sa_raw[i] = 0x3c003c00u;
        if (g.c_f16) {
#pragma unroll
            for (int bj = 0; bj < WN; ++bj) {
                const int64_t n = n_lane + bj * 32;
                const uint32_t h = (g.w_scale && n < g.N) ? g.w_scale[n] : 0x3c00u;
                sw_raw[bj / 2] = (bj & 1) ? (sw_raw[bj / 2] & 0xffffu) | (h << 16) : (sw_raw[bj / 2] & 0xffff0000u) | h;
            }
#pragma unroll
            for (int i = 0; i < (WM + 1) / 2; ++i) {
                const int64_t m = m0 + wave_m * WM * 32 + lane + 64 * i;
                const uint32_t h = (g.a_scale && m < g.M && lane + 64 * i < 32 * WM) ? g.a_scale[m] : 0x3c00u;
                sa_raw[i / 2] = (i & 1) ? (sa_raw[i / 2] & 0xffffu) | (h << 16) : (sa_raw[i / 2] & 0xffff0000u) | h;
            }
        }
    }

    auto init_phase = [&](auto ph_c) __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_c)::value;
        constexpr int WMP = split_rows(WM, SPLIT, ph), ROW0 = split_row0(WM, SPLIT, ph);
        v16f zero;
#pragma unroll
        for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
        for (int bi = 0; bi < WMP; ++bi) {
            float a_in;
            if constexpr (PRELOAD) {
                a_in = a_init[ROW0 + bi];
            } else {  // loaded here, block by block: no register to spare for holding them
                int64_t m = m0 + (wave_m * WM + ROW0 + bi) * 32 + r32;
                if (m >= rows_a) m = rows_a - 1;
                const float rt = -(float)(2u * cw * (uint32_t)g.a_sum[m]);
                a_in = kh == 0 ? rt : 1.0f;
            }
#pragma unroll
            for (int bj = 0; bj < WN; ++bj)
                acc[ROW0 + bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_in, b_init[bj], zero, 0, 0, 0);
        }
    };

    // int32 store of element e of phase ph under the k loop of the next phase: elements run along the row
    // blocks, then the 16 registers (rows), then the column blocks, so that the row pointer moves once per WN stores
    const int64_t row_bytes = g.N * 4;
    char *st_ptr = nullptr;
    auto store_elem = [&](auto ph_c, auto e_c) __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_c)::value, e = decltype(e_c)::value;
        constexpr int bi = split_row0(WM, SPLIT, ph) + e / (16 * WN), v = (e / WN) % 16, bj = e % WN;
        // rows of consecutive registers: +1, +1, +1, +5 (the next group of four rows, or the next row block)
        if constexpr (bj == 0 && e > 0) st_ptr += (v % 4 == 0 ? 5 : 1) * row_bytes;
        // streaming store: the output is not read again, and keeping it out of the way of the operand tiles in
        // L2 (and written back early rather than at the end of the kernel) is worth about 5 % at 4096^2 outputs
        __builtin_nontemporal_store((int32_t)acc[bi][bj][v], reinterpret_cast<int32_t *>(st_ptr + bj * 128));
    };

    // One sweep of K for phase ph, the activation group at slot slot_a and the weight group at slot slot_b
    // (AS / BS: the group is a single one).  exp_a + exp_b - 254 = 4 + the bit positions of the two groups.
    // STORES: the first STORE_STAGES stages also store phase ph - 1.
    // PRELOADED: stage 0 is already in buffer 0 (the prologue's request).
    auto sweep = [&](auto ph_c, auto stores_c, auto as_c, auto bs_c, int slot_a, int slot_b, int exp_a, int exp_b,
                     auto preloaded_c) __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_c)::value;
        constexpr bool STORES = decltype(stores_c)::value, PRELOADED = decltype(preloaded_c)::value;
        constexpr bool AS = decltype(as_c)::value, BS = decltype(bs_c)::value;
        constexpr int WMP = split_rows(WM, SPLIT, ph), ROW0 = split_row0(WM, SPLIT, ph);  // this phase's row blocks
        constexpr int PER_KS = WMP * WN;         // MFMAs per k step
        constexpr int FRAG0 = AF ? WMP : 0;      // first fragment that needs expanding (A blocks come first)
        constexpr int FRAGS = WMP + WN;          // operand fragments per k step
        constexpr int TASKS = 4 * (FRAGS - FRAG0);  // expansion dwords per k step
        constexpr int TPM = (TASKS + PER_KS - 1) / PER_KS;  // tasks per MFMA (the last MFMAs of a step may get fewer)
        constexpr int STAGE_ELEMS = KS * PER_KS / STORE_EVERY;  // outputs of the previous phase stored under one stage
        auto load_stage = [&](auto buf_c, int64_t st) __attribute__((always_inline)) {
            load_stage_of(ph_c, as_c, bs_c, buf_c, st, slot_a, slot_b);
        };
        // dword d of fragment f (f < WMP: A block f, else B block f - WMP) of k step ks, from buffer buf
        auto expand = [&](auto buf_c, auto ks_c, auto f_c, auto d_c) __attribute__((always_inline)) {
            constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value, f = decltype(f_c)::value,
                          d = decltype(d_c)::value;
            if constexpr (f < WMP) {
                if constexpr (AF) {
                    // nothing to expand
                } else if constexpr (AS) {
                    af[ks & 1][f][d] = (int)fp4_single_dword<ks, d>(ra[buf][f][0]);
                } else {
                    af[ks & 1][f][d] = (int)fp4_pair_dword<ks, d>(ra[buf][f][0], ra[buf][f][1]);
                }
            } else {
                if constexpr (BS) bf[ks & 1][f - WMP][d] = (int)fp4_single_dword<ks, d>(rb[buf][f - WMP][0]);
                else bf[ks & 1][f - WMP][d] = (int)fp4_pair_dword<ks, d>(rb[buf][f - WMP][0], rb[buf][f - WMP][1]);
            }
        };
        // one stage with its raw words in buffer `buf`; loads stage st+1 (clamped) into the other buffer;
        // chunk >= 0: stores elements chunk * STAGE_ELEMS ... of the previous phase on the way
        auto stage = [&](auto buf_c, int64_t st, auto chunk_c) __attribute__((always_inline)) {
            constexpr int buf = decltype(buf_c)::value, chunk = decltype(chunk_c)::value;
            using Other = std::integral_constant<int, buf ^ 1>;
            load_stage(Other{}, st + 1 < nst ? st + 1 : st);  // the surplus load of the last stage is discarded
            __builtin_amdgcn_sched_barrier(0);
            static_for<KS * PER_KS>([&](auto i_c) __attribute__((always_inline)) {
                constexpr int i = decltype(i_c)::value;
                constexpr int ks = i / PER_KS, j = i % PER_KS, bi = j / WN, bj = j % WN;
                const v4i b = bf[ks & 1][bj];
                const v8i b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
                // operand formats: 4 = E2M1, 2 = E2M3; the scales are E8M0 exponents (127 = 2^0)
                if constexpr (AF) {
                    // words 6 ks .. 6 ks + 5 of the lane's 24 raw words
                    auto raw = [&](auto w_c) __attribute__((always_inline)) {
                        constexpr int w = 6 * ks + decltype(w_c)::value;
                        return (int)vec_word<w & 3>(ra[buf][bi][w >> 2]);
                    };
                    const v8i a8 = {raw(std::integral_constant<int, 0>{}), raw(std::integral_constant<int, 1>{}),
                                    raw(std::integral_constant<int, 2>{}), raw(std::integral_constant<int, 3>{}),
                                    raw(std::integral_constant<int, 4>{}), raw(std::integral_constant<int, 5>{}), 0, 0};
                    acc[ROW0 + bi][bj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        a8, b8, acc[ROW0 + bi][bj], 2, 4, 0, exp_a, 0, exp_b + (BS ? fp4_single_exponent(ks) : 0));
                } else {
                    const v4i a = af[ks & 1][bi];
                    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
                    acc[ROW0 + bi][bj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        a8, b8, acc[ROW0 + bi][bj], 4, 4, 0, exp_a + (AS ? fp4_single_exponent(ks) : 0), 0,
                        exp_b + (BS ? fp4_single_exponent(ks) : 0));
                }
                // this MFMA's share of the next k step's operands (after the last step: step 0 of stage st+1)
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
                if constexpr (chunk >= 0 && i % STORE_EVERY == 0)
                    store_elem(std::integral_constant<int, (ph > 0 ? ph - 1 : 0)>{},
                               std::integral_constant<int, chunk * STAGE_ELEMS + i / STORE_EVERY>{});
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        if constexpr (!PRELOADED) load_stage(I0{}, 0);
        // fragments of (stage 0, k step 0)
        static_for<FRAGS - FRAG0>([&](auto f_c) __attribute__((always_inline)) {
            using F = std::integral_constant<int, FRAG0 + decltype(f_c)::value>;
            static_for<4>([&](auto d_c) __attribute__((always_inline)) { expand(I0{}, I0{}, F{}, d_c); });
        });
        int64_t st = 0;
        if constexpr (STORES) {
            static_for<STORE_STAGES / 2>([&](auto h_c) __attribute__((always_inline)) {
                constexpr int h = decltype(h_c)::value;
                stage(I0{}, 2 * h, std::integral_constant<int, 2 * h>{});
                stage(I1{}, 2 * h + 1, std::integral_constant<int, 2 * h + 1>{});
            });
            st = STORE_STAGES;
        }
        for (; st < nst; st += 2) {
            stage(I0{}, st, NoStore{});
            stage(I1{}, st + 1, NoStore{});
        }
    };

    using T = std::true_type;
    using F = std::false_type;
    static_for<PHASES>([&](auto ph_c) __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_c)::value;
        init_phase(ph_c);
        if constexpr (ph > 0)  // row pointer of element 0 of the previous phase
            st_ptr = reinterpret_cast<char *>(g.c_i32 + (m_lane + split_row0(WM, SPLIT, ph - 1) * 32) * g.N + n_lane);
        // the first sweep of a later phase carries the stores of the phase before it
        using First = std::integral_constant<bool, (ph > 0)>;
        using Pre = std::integral_constant<bool, (ph == 0 && PRELOAD)>;  // stage 0 of the very first sweep came with the prologue
        if constexpr (AF) {
            // one sweep per weight group; (ua / 8)(uw / 2) 2^6 = 4 ua uw
            if constexpr (pair_groups(Q) > 0) {
                sweep(ph_c, First{}, F{}, F{}, 0, 0, 130, 130, Pre{});
                for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(ph_c, F{}, F{}, F{}, 0, 2 * hb, 130, 130 + 2 * hb, F{});
                if constexpr (has_single_group(Q)) sweep(ph_c, F{}, F{}, T{}, 0, Q - 1, 130, 130 + Q - 1, F{});
            } else {
                sweep(ph_c, First{}, F{}, T{}, 0, 0, 130, 130, Pre{});
            }
        } else
        // pair x pair, pair x single, single x pair, single x single
        if constexpr (pair_groups(P) > 0) {
            if constexpr (pair_groups(Q) > 0) {
                sweep(ph_c, First{}, F{}, F{}, 0, 0, 129, 129, Pre{});
                for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(ph_c, F{}, F{}, F{}, 0, 2 * hb, 129, 129 + 2 * hb, F{});
                if constexpr (has_single_group(Q)) sweep(ph_c, F{}, F{}, T{}, 0, Q - 1, 129, 129 + Q - 1, F{});
            } else {
                sweep(ph_c, First{}, F{}, T{}, 0, Q - 1, 129, 129 + Q - 1, Pre{});
            }
            for (int ha = 1; ha < pair_groups(P); ++ha) {
                for (int hb = 0; hb < pair_groups(Q); ++hb)
                    sweep(ph_c, F{}, F{}, F{}, 2 * ha, 2 * hb, 129 + 2 * ha, 129 + 2 * hb, F{});
                if constexpr (has_single_group(Q)) sweep(ph_c, F{}, F{}, T{}, 2 * ha, Q - 1, 129 + 2 * ha, 129 + Q - 1, F{});
            }
            if constexpr (has_single_group(P)) {
                for (int hb = 0; hb < pair_groups(Q); ++hb)
                    sweep(ph_c, F{}, T{}, F{}, P - 1, 2 * hb, 129 + P - 1, 129 + 2 * hb, F{});
                if constexpr (has_single_group(Q)) sweep(ph_c, F{}, T{}, T{}, P - 1, Q - 1, 129 + P - 1, 129 + Q - 1, F{});
            }
        } else {  // P == 1
            if constexpr (pair_groups(Q) > 0) {
                sweep(ph_c, First{}, T{}, F{}, 0, 0, 129, 129, Pre{});
                for (int hb = 1; hb < pair_groups(Q); ++hb) sweep(ph_c, F{}, T{}, F{}, 0, 2 * hb, 129, 129 + 2 * hb, F{});
                if constexpr (has_single_group(Q)) sweep(ph_c, F{}, T{}, T{}, 0, Q - 1, 129, 129 + Q - 1, F{});
            } else {
                sweep(ph_c, First{}, T{}, T{}, 0, 0, 129, 129, Pre{});
            }
        }
    });

    // Store of the last phase.  The output mode and the border test are uniform over the workgroup, so
    // straight-line store sequences are chosen per output instead of testing per element.
    constexpr int LAST = PHASES - 1;
    constexpr int WML = split_rows(WM, SPLIT, LAST), ROWL = split_row0(WM, SPLIT, LAST);  // row blocks of the last phase
    const int64_t m_last = m_lane + ROWL * 32;
    // PAIR (interior tiles, even N, 4-byte aligned fp16 output): neighbouring lanes hold neighbouring columns,
    // and a 2-byte store per lane writes 64-byte runs, which the memory system handles far worse than 128-byte
    // runs (a 16 MiB fp16 output cost 7 us that way).  Rows are taken in pairs: the even lane of a lane pair
    // collects both columns of the first row, the odd lane both columns of the second row (one lane exchange),
    // and each stores one dword.
    // NT (interior tiles, a single output): streaming stores.  They gain 3 - 15 % when one output is written (more
    // the larger the output), and lose as much when the int32 and the fp16 pass follow each other.
    auto emit = [&](auto guard_c, auto i32_c, auto f16_c, auto pair_c, auto nt_c) __attribute__((always_inline)) {
        constexpr bool GUARD = decltype(guard_c)::value, I32 = decltype(i32_c)::value, F16 = decltype(f16_c)::value,
                       PAIR = decltype(pair_c)::value, NT = decltype(nt_c)::value;
        int32_t *ci = I32 ? g.c_i32 + m_last * g.N + n_lane : nullptr;
        uint16_t *ch = F16 ? g.c_f16 + m_last * g.N + n_lane : nullptr;
        const bool odd = lane & 1;
        // odd lanes write the row below at the column to the left
        uint16_t *ch_pair = F16 ? ch + (odd ? g.N - 1 : 0) : nullptr;
        // token scale of row (block bi of the last phase, register v) of this lane, from the lane that loaded it
        auto token_scale = [&](int bi, int v) __attribute__((always_inline)) {
            const int blk = ROWL + bi;  // row block inside the wave tile: rows 64 (blk / 2) + lane were loaded
            const int src = (blk & 1) * 32 + 8 * (v / 4) + 4 * kh + (v % 4);
            const uint32_t both = (uint32_t)__shfl((int)sa_raw[blk / 4], src);
            return half_bits_to_float((uint16_t)((blk / 2) & 1 ? both >> 16 : both & 0xffffu));
        };
        float sw[WN];
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
            sw[bj] = half_bits_to_float((uint16_t)((bj & 1) ? sw_raw[bj / 2] >> 16 : sw_raw[bj / 2] & 0xffffu));
#pragma unroll
        for (int bi = 0; bi < WML; ++bi) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = (int64_t)(bi * 32 + 8 * (v / 4) + (v % 4));  // relative to m_last
                // the lane permutes come before any lane leaves the iteration: a lane that has left supplies nothing
                const float sa = F16 ? token_scale(bi, v) : 1.0f;
                const float sa_next = (F16 && PAIR && v % 2 == 0) ? token_scale(bi, v + 1) : 1.0f;
                if (GUARD && m_last + row >= g.M) continue;
#pragma unroll
                for (int bj = 0; bj < WN; ++bj) {
                    if (GUARD && n_lane + bj * 32 >= g.N) continue;
                    const float c = acc[ROWL + bi][bj][v];  // = C, an integer
                    if constexpr (I32 && NT) __builtin_nontemporal_store((int32_t)c, &ci[row * g.N + bj * 32]);
                    if constexpr (I32 && !NT) ci[row * g.N + bj * 32] = (int32_t)c;
                    if constexpr (F16 && !PAIR) ch[row * g.N + bj * 32] = float_to_half_bits(c * sa * sw[bj]);
                    if constexpr (F16 && PAIR) {
                        if (v % 2 == 0) {  // folds once the loop is unrolled
                            const uint32_t h0 = float_to_half_bits(c * sa * sw[bj]);
                            const uint32_t h1 = float_to_half_bits(acc[ROWL + bi][bj][(v + 1) & 15] * sa_next * sw[bj]);
                            const uint32_t give = odd ? h0 : h1, keep = odd ? h1 : h0;
                            // quad_perm [1, 0, 3, 2]: the value of the other lane of the pair
                            const uint32_t got = (uint32_t)__builtin_amdgcn_mov_dpp((int)give, 0xB1, 0xf, 0xf, true);
                            const uint32_t word = odd ? (got | (keep << 16)) : (keep | (got << 16));
                            uint32_t *dst = reinterpret_cast<uint32_t *>(ch_pair + row * g.N + bj * 32);
                            if constexpr (NT) __builtin_nontemporal_store(word, dst);
                            else *dst = word;
                        }
                    }
                }
            }
        }
    };
    if constexpr (PHASES > 1) {
        emit(F{}, T{}, F{}, F{}, T{});  // interior tiles, int32 output only (checked by the launcher)
    } else {
        const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N);
        const bool pair = (g.N & 1) == 0 && (reinterpret_cast<uintptr_t>(g.c_f16) & 3u) == 0;
        const bool single = !(g.c_i32 && g.c_f16);
        // both outputs: one pass per output (a combined pass needs more registers than there are)
        if (g.c_i32) {
            if (interior && single) emit(F{}, T{}, F{}, F{}, T{});
            else if (interior) emit(F{}, T{}, F{}, F{}, F{});
            else emit(T{}, T{}, F{}, F{}, F{});
        }
        if (g.c_f16) {
            if (interior && pair && single) emit(F{}, F{}, T{}, T{}, T{});
            else if (interior && pair) emit(F{}, F{}, T{}, T{}, F{});
            else if (interior) emit(F{}, F{}, T{}, F{}, F{});
            else emit(T{}, F{}, T{}, F{}, F{});
        }
    }
}

// The split kernels store int32 only and need whole tiles and enough stages of K to carry the stores.
template <int P, int Q, int WM, int WN, int SPLIT>
inline bool direct_split_usable(const GemmArgs &g)
{
    const int64_t nst = g.nkb / 2;
    return g.c_i32 && !g.c_f16 && g.M % (64 * WM) == 0 && g.N % (64 * WN) == 0 &&
           nst >= split_store_stages(WM, WN, SPLIT);
}

template <int P, int Q, int WM, int WN, int SPLIT = 1>
hipError_t launch_direct_variant(const GemmArgs &g, hipStream_t stream)
{
    constexpr int BM = 32 * WM * waves_m(WM), BN = 32 * WN * waves_n(WM);
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int64_t tiles = tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL || g.M > 0x7fffffffLL || g.N > 0x7fffffffLL || g.K > 0x7fffffffLL) return hipErrorInvalidValue;
    const KernelTiming timing = take_kernel_timing();
    note_kernel("gemm_mfma_direct_kernel<%d,%d,%d,%d,%d>", P, Q, WM, WN, SPLIT);
    if (timing.start || timing.stop)
        hipExtLaunchKernelGGL((gemm_mfma_direct_kernel<P, Q, WM, WN, SPLIT>), dim3((unsigned)tiles), dim3(256), 0,
                              stream, timing.start, timing.stop, 0, g.a, g.w, g.c_i32, g.c_f16, (int)g.M, (int)g.N, (int)g.K,
                              (int)g.nkb, (int)tiles_n, (int)tiles, g.w_scale, g.a_scale);
    else
        hipLaunchKernelGGL((gemm_mfma_direct_kernel<P, Q, WM, WN, SPLIT>), dim3((unsigned)tiles), dim3(256), 0,
                           stream, g.a, g.w, g.c_i32, g.c_f16, (int)g.M, (int)g.N, (int)g.K, (int)g.nkb, (int)tiles_n,
                           (int)tiles, g.w_scale, g.a_scale);
    return hipGetLastError();
}

}  // namespace mfma
}  // namespace apmm
