// Ablation kernels for the claim of paper Sec. 4.2 (evidence, not the product path; reachable through
// apmm_gemm_ex with their own algo ids).  The paper argues that computing every 1-bit plane pair as a
// MatMul of its own and recovering C = sum_ij 2^(i+j) D_ij in global memory wastes the time on memory
// traffic, and keeps the plane products of a tile on chip instead (recovery in fragments / shared memory).
// Both schemes are built here on the matrix unit of gfx950, with the planes as +-1 operands:
//
//   gemm_mfma_planes_kernel<P, Q, true>  + recover_planes_kernel   ("naive"): one plane pair (i, j) per
//       workgroup; its 32-bit product D_ij goes to global memory (p q matrices of M x N int32); a second
//       pass reads all of them, shifts, adds and stores C.
//   gemm_mfma_planes_kernel<P, Q, false>                            ("planes in registers"): one output tile
//       per workgroup; for every weight plane i one sweep of K with an accumulator per activation plane j,
//       then C += D_ij << (i + j) in registers; only C reaches global memory.
//
// Operands: a plane bit b is the value 2b - 1 (paper Eq. 1); as an E2M1 nibble that is 0010 (+1) or 1010 (-1),
// made from the packed words of apmm_layout.h with two operations per dword (shift the inverted bit to the
// sign position, insert the constant).  v_mfma_scale_f32_32x32x64_f8f6f4 then gives D_ij directly, exact in
// fp32 (|D_ij| <= K).  Padded k positions hold set bits in both operands: +1 each, subtracted at the end.
// Same tile map and operand loads as the product kernel (apmm_gemm_mfma_direct.h): 128 x 128 tile, 2 x 2 waves
// of 64 x 64, lane l owns row l % 32 and k block l / 32 of a two-block stage, raw words double buffered in
// registers.  Activations of 1 or 2 bits only (wider ones are stored in the field form).
#include "apmm_mfma_common.h"

namespace apmm {
namespace {

using mfma::v16f;
using mfma::v8i;

// E2M1 dword D of k step KS with the +-1 values of one plane.  PAIR: the plane is bit `b` of a pair group held as
// u0 = S[0..3], u1 = S[4..7]; else the single group L[0..3] in u0.  nu0 / nu1 are the inverted words.
template <bool SINGLE, int KS, int D>
__device__ __forceinline__ uint32_t plane_dword(const uint4 &nu0, const uint4 &nu1, int b)
{
    // bit position of the plane inside the nibble: single group KS, pair group 2 tt + b (tt = D % 2)
    const uint32_t w = SINGLE ? mfma::vec_word<D>(nu0) : mfma::pair_word<2 * KS + D / 2>(nu0, nu1);
    const int pos = SINGLE ? KS : 2 * (D & 1) + b;
    return ((w << (3 - pos)) & 0x88888888u) | 0x22222222u;  // sign = inverted bit, magnitude 1.0
}

template <int P, int Q, bool NAIVE>
__global__ __launch_bounds__(256) void gemm_mfma_planes_kernel(GemmArgs g, int32_t *__restrict__ pairs_out, int tiles_n,
                                                               int tiles_total)
{
    static_assert(P >= 1 && P <= 2 && Q >= 1 && Q <= 4, "activations in the group form, weights up to four bits");
    constexpr int WM = 2, WN = 2, BM = 128, BN = 128, KS = 4;
    constexpr bool AS = P == 1;                 // the activation planes: one single group, or the two bits of a pair group
    constexpr int PJ = NAIVE ? 1 : P;           // activation planes multiplied per sweep
    constexpr int kSlotVec = kPlaneWords / 4;
    constexpr int kStageVecA = 2 * P * kSlotVec, kStageVecB = 2 * Q * kSlotVec;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1, r32 = lane & 31, kh = lane >> 5;
    const int lid = mfma::xcd_tile_id(blockIdx.x, tiles_total);
    const int tm = lid / tiles_n, tn = lid % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
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
    const int64_t nst = g.nkb / 2;
    const int32_t pad = (int32_t)(g.nkb * kKBlock - g.K);  // padded k positions: +1 in every plane pair

    int32_t c_acc[WM][WN][16];  // the recovered result (planes in registers)
#pragma unroll
    for (int bi = 0; bi < WM; ++bi)
#pragma unroll
        for (int bj = 0; bj < WN; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) c_acc[bi][bj][v] = 0;

    // One sweep of K for weight plane `i` (bit `bb` of the group at slot `slot_b`, BS: a single group) against
    // the activation planes j0 .. j0 + PJ - 1; afterwards `fold` gets each D_ij.
    auto sweep = [&](auto bs_c, int slot_b, int bb, int j0, auto &&fold) __attribute__((always_inline)) {
        constexpr bool BS = decltype(bs_c)::value;
        v16f acc[PJ][WM][WN];
#pragma unroll
        for (int j = 0; j < PJ; ++j)
#pragma unroll
            for (int bi = 0; bi < WM; ++bi)
#pragma unroll
                for (int bj = 0; bj < WN; ++bj)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[j][bi][bj][v] = 0.f;
        uint4 ra[2][WM][2], rb[2][WN][2];  // raw words by stage parity
        auto load_stage = [&](int buf, int64_t st) __attribute__((always_inline)) {
#pragma unroll
            for (int bi = 0; bi < WM; ++bi) {
                ra[buf][bi][0] = pa_src[bi][st * kStageVecA];
                if constexpr (!AS) ra[buf][bi][1] = pa_src[bi][st * kStageVecA + kSlotVec];
            }
#pragma unroll
            for (int bj = 0; bj < WN; ++bj) {
                rb[buf][bj][0] = pb_src[bj][st * kStageVecB + slot_b * kSlotVec];
                if constexpr (!BS) rb[buf][bj][1] = pb_src[bj][st * kStageVecB + (slot_b + 1) * kSlotVec];
            }
        };
        auto invert = [](uint4 u) { return make_uint4(~u.x, ~u.y, ~u.z, ~u.w); };
        auto stage = [&](auto buf_c, int64_t st) __attribute__((always_inline)) {
            constexpr int buf = decltype(buf_c)::value;
            load_stage(buf ^ 1, st + 1 < nst ? st + 1 : st);  // the surplus load of the last stage is discarded
            uint4 na[WM][2], nb[WN][2];
#pragma unroll
            for (int bi = 0; bi < WM; ++bi) {
                na[bi][0] = invert(ra[buf][bi][0]);
                na[bi][1] = AS ? na[bi][0] : invert(ra[buf][bi][1]);
            }
#pragma unroll
            for (int bj = 0; bj < WN; ++bj) {
                nb[bj][0] = invert(rb[buf][bj][0]);
                nb[bj][1] = BS ? nb[bj][0] : invert(rb[buf][bj][1]);
            }
            mfma::static_for<KS>([&](auto ks_c) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_c)::value;
                v8i b8[WN];
#pragma unroll
                for (int bj = 0; bj < WN; ++bj) {
                    b8[bj] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
                    mfma::static_for<4>([&](auto d_c) __attribute__((always_inline)) {
                        constexpr int d = decltype(d_c)::value;
                        b8[bj][d] = (int)plane_dword<BS, ks, d>(nb[bj][0], nb[bj][1], bb);
                    });
                }
#pragma unroll
                for (int j = 0; j < PJ; ++j) {
#pragma unroll
                    for (int bi = 0; bi < WM; ++bi) {
                        v8i a8 = {0, 0, 0, 0, 0, 0, 0, 0};
                        mfma::static_for<4>([&](auto d_c) __attribute__((always_inline)) {
                            constexpr int d = decltype(d_c)::value;
                            a8[d] = (int)plane_dword<AS, ks, d>(na[bi][0], na[bi][1], j0 + j);
                        });
#pragma unroll
                        for (int bj = 0; bj < WN; ++bj)  // operand formats 4 = E2M1, scales 2^0
                            acc[j][bi][bj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8[bj], acc[j][bi][bj], 4, 4,
                                                                                            0, 127, 0, 127);
                    }
                }
            });
        };
        load_stage(0, 0);
        for (int64_t st = 0; st < nst; st += 2) {  // the packed K is a multiple of 512: an even number of stages
            stage(std::integral_constant<int, 0>{}, st);
            stage(std::integral_constant<int, 1>{}, st + 1);
        }
#pragma unroll
        for (int j = 0; j < PJ; ++j) fold(j0 + j, acc[j]);
    };
    // weight plane i: bit b of the pair group at slots 2 (i / 2), 2 (i / 2) + 1, or the single group at slot Q - 1
    auto sweep_plane = [&](int i, int j0, auto &&fold) __attribute__((always_inline)) {
        if (i < 2 * pair_groups(Q)) sweep(std::false_type{}, 2 * (i / 2), i & 1, j0, fold);
        else sweep(std::true_type{}, Q - 1, 0, j0, fold);
    };

    // Accumulator layout of the 32x32 MFMA: lane l, register v holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32.
    const int64_t m_lane = m0 + wave_m * WM * 32 + kh * 4, n_lane = n0 + wave_n * WN * 32 + r32;
    if constexpr (NAIVE) {
        // this workgroup's plane pair: its product goes to global memory as it is
        const int pair = (int)blockIdx.y, i = pair / P, j = pair % P;
        int32_t *out = pairs_out + (int64_t)pair * g.M * g.N;
        sweep_plane(i, j, [&](int, v16f (&d)[WM][WN]) __attribute__((always_inline)) {
#pragma unroll
            for (int bi = 0; bi < WM; ++bi)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t m = m_lane + bi * 32 + 8 * (v / 4) + (v % 4);
                    if (m >= g.M) continue;
#pragma unroll
                    for (int bj = 0; bj < WN; ++bj) {
                        const int64_t n = n_lane + bj * 32;
                        if (n < g.N) out[m * g.N + n] = (int32_t)d[bi][bj][v] - pad;
                    }
                }
        });
    } else {
        for (int i = 0; i < Q; ++i) {
            sweep_plane(i, 0, [&](int j, v16f (&d)[WM][WN]) __attribute__((always_inline)) {
                // paper Sec. 3.2 step 3, in registers: C += D_ij << (i + j)
#pragma unroll
                for (int bi = 0; bi < WM; ++bi)
#pragma unroll
                    for (int bj = 0; bj < WN; ++bj)
#pragma unroll
                        for (int v = 0; v < 16; ++v) c_acc[bi][bj][v] += ((int32_t)d[bi][bj][v] - pad) << (i + j);
            });
        }
#pragma unroll
        for (int bi = 0; bi < WM; ++bi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m_lane + bi * 32 + 8 * (v / 4) + (v % 4);
                if (m >= g.M) continue;
                const float sa = load_scale(g.a_scale, m);
#pragma unroll
                for (int bj = 0; bj < WN; ++bj) {
                    const int64_t n = n_lane + bj * 32;
                    if (n < g.N) store_output(g, m, n, c_acc[bi][bj][v], sa, load_scale(g.w_scale, n));
                }
            }
    }
}

// Second pass of the naive scheme (paper Sec. 3.2 step 3, in global memory): C = sum_ij D_ij << (i + j) over the
// p q product matrices, four consecutive outputs per thread where the row length allows 16-byte accesses.
__global__ __launch_bounds__(256) void recover_planes_kernel(GemmArgs g, const int32_t *__restrict__ pairs, bool vec4)
{
    const int64_t total = g.M * g.N, per = vec4 ? 4 : 1;
    const int64_t first = ((int64_t)blockIdx.x * 256 + threadIdx.x) * per;
    if (first >= total) return;
    int32_t c[4] = {0, 0, 0, 0};
    for (int i = 0; i < g.q; ++i)
        for (int j = 0; j < g.p; ++j) {
            const int32_t *d = pairs + (int64_t)(i * g.p + j) * total + first;
            if (vec4) {
                const int4 v = *reinterpret_cast<const int4 *>(d);
                c[0] += v.x << (i + j); c[1] += v.y << (i + j); c[2] += v.z << (i + j); c[3] += v.w << (i + j);
            } else {
                c[0] += d[0] << (i + j);
            }
        }
    for (int e = 0; e < per; ++e) {
        const int64_t at = first + e, m = at / g.N, n = at % g.N;
        store_output(g, m, n, c[e], load_scale(g.a_scale, m), load_scale(g.w_scale, n));
    }
}

template <int P, int Q>
hipError_t launch_planes(const GemmArgs &g, int32_t *pairs, hipStream_t stream)
{
    const int64_t tiles_m = (g.M + 127) / 128, tiles_n = (g.N + 127) / 128, tiles = tiles_m * tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    if (pairs) {
        note_kernel("gemm_mfma_planes_kernel<%d,%d,pairs to global memory> + recover_planes_kernel", P, Q);
        hipLaunchKernelGGL((gemm_mfma_planes_kernel<P, Q, true>), dim3((unsigned)tiles, P * Q), dim3(256), 0, stream, g, pairs,
                           (int)tiles_n, (int)tiles);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const int64_t total = g.M * g.N;
        const bool vec4 = (g.N & 3) == 0 && (reinterpret_cast<uintptr_t>(pairs) & 15) == 0;
        const int64_t threads = vec4 ? total / 4 : total;
        const int64_t blocks = (threads + 255) / 256;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(recover_planes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, g, pairs, vec4);
        return hipGetLastError();
    }
    note_kernel("gemm_mfma_planes_kernel<%d,%d,recovery in registers>", P, Q);
    hipLaunchKernelGGL((gemm_mfma_planes_kernel<P, Q, false>), dim3((unsigned)tiles), dim3(256), 0, stream, g, nullptr,
                       (int)tiles_n, (int)tiles);
    return hipGetLastError();
}

template <int P>
hipError_t launch_planes_p(const GemmArgs &g, int32_t *pairs, hipStream_t stream)
{
    switch (g.q) {
    case 1: return launch_planes<P, 1>(g, pairs, stream);
    case 2: return launch_planes<P, 2>(g, pairs, stream);
    case 3: return launch_planes<P, 3>(g, pairs, stream);
    case 4: return launch_planes<P, 4>(g, pairs, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

// 1- or 2-bit activations, weights of up to 4 bits, every D_ij and every partial sum of the recovery below 2^24
// (fp32 accumulators; the same bound as the product kernel).
bool gemm_ablation_supported(const GemmArgs &g)
{
    if (g.p < 1 || g.p > 2 || g.q < 1 || g.q > 4) return false;
    const int64_t unit = (int64_t)((1 << g.p) - 1) * ((1 << g.q) - 1);
    return 4 * g.nkb * kKBlock * unit < (1 << 24);
}

size_t gemm_ablation_pairs_bytes(const GemmArgs &g) { return (size_t)g.p * g.q * (size_t)g.M * (size_t)g.N * 4u; }

hipError_t launch_gemm_ablation(const GemmArgs &g, int32_t *pairs, hipStream_t stream)
{
    return g.p == 1 ? launch_planes_p<1>(g, pairs, stream) : launch_planes_p<2>(g, pairs, stream);
}

}  // namespace apmm
