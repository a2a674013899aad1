// Pieces shared by the MFMA GEMM kernels: compile-time loops, the plane -> operand expansion,
// the two operand formats and the tile store with the recovery terms.
#pragma once
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "apmm_epilogue.h"
#include "apmm_kernels.h"

namespace apmm {
namespace mfma {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

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

// Output dword t of the expansion of one 32-element group given its planes w[0..NB-1].
// Plane i is stored rotated left by i (apmm_layout.h).
//   INT8: dword t of 8 holds 4 codes as bytes; their plane-i bits are at in-byte position (t+i) % 8.
//   FP4 : dword t of 4 holds 8 codes as nibbles; their plane-i bits are at in-nibble position (t+i) % 4.
// One rotate right by t brings every plane to its own bit i of the byte / nibble.
template <int NB, bool FP4>
__device__ __forceinline__ uint32_t expand_dword(const uint32_t (&w)[NB], int t)
{
    constexpr uint32_t ones = FP4 ? 0x11111111u : 0x01010101u;
    constexpr int period = FP4 ? 4 : 8;
    uint32_t y = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) y |= w[i] & (ones << ((t + i) % period));
    return t ? __builtin_rotateright32(y, t) : y;
}

// The same for a group of NB planes that starts at plane index `first` (uniform at run time): the
// planes of the group are rotated by first + i, so the masks move by `first` and the final rotate
// brings plane first + i to bit i of the nibble.  FP4 only.
template <int NB>
__device__ __forceinline__ uint32_t expand_group_dword(const uint32_t (&w)[NB], int t, int first)
{
    uint32_t y = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) y |= w[i] & (0x11111111u << ((t + i + first) & 3));
    return __builtin_rotateright32(y, (t + first) & 31);
}

// The two operand formats of the matrix unit.
//   INT8: code u as a byte, v_mfma_i32_32x32x32_i8, int32 accumulate: acc = S.
//   FP4 : code u as the E2M1 pattern 00uu = u/2, v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales,
//         fp32 accumulate: acc = S/4 exactly (every product is a multiple of 1/4, every partial sum
//         is representable for K <= 2^20).
template <bool FP4>
struct Acc;
template <>
struct Acc<false> {
    typedef v16i type;
    static __device__ __forceinline__ type mma(v4i a, v4i b, type c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
    // 4 S as a wrapping 32-bit integer
    static __device__ __forceinline__ uint32_t four_s(int v) { return (uint32_t)v << 2; }
};
template <>
struct Acc<true> {
    typedef v16f type;
    static __device__ __forceinline__ type mma(v4i a, v4i b, type c)
    {
        const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
        // formats 4 / 4 = E2M1 for both operands; scale exponent 127 = 2^0
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 127, 0, 127);
    }
    // the same with the A operand scaled by 2^(scale_a - 127) (E8M0 exponent, read from byte 0)
    static __device__ __forceinline__ type mma_scaled(v4i a, v4i b, type c, int scale_a)
    {
        const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, scale_a, 0, 127);
    }
    static __device__ __forceinline__ uint32_t four_s(float v) { return (uint32_t)(int32_t)(v * 16.0f); }
};

// Store of one wave's (32*WM) x (32*WN) accumulator tile with the recovery
//   C = 4 S - 2 cw PA[m] - 2 ca PW[n] + K ca cw        (wrapping 32-bit arithmetic; C itself fits)
// and the optional fp16 scale epilogue.
//   m_lane, n_lane : global row of (bi = 0, v4 = 0, r = 0) and global column of bj = 0 for this lane
//   pa4(bi, v4)    : PA of the four consecutive rows m_lane + 32 bi + 8 v4 + (0..3), as int4
//   pw[bj]         : PW of column n_lane + 32 bj
// Accumulator layout of the 32x32 MFMA: lane l, register v holds row 8*(v/4) + 4*(l/32) + v%4,
// column l%32.  The output mode and the border test are uniform over the workgroup, so one of six
// straight-line store sequences is chosen instead of testing per element.
template <int P, int Q, int WM, int WN, bool FP4, class PA4>
__device__ __forceinline__ void store_wave_tile(const GemmArgs &g, const typename Acc<FP4>::type (&acc)[WM][WN],
                                                int64_t m_lane, int64_t n_lane, bool interior, PA4 &&pa4,
                                                const uint32_t (&pw)[WN])
{
    constexpr uint32_t ca = (1u << P) - 1, cw = (1u << Q) - 1;
    const uint32_t base = (uint32_t)g.K * ca * cw;
    uint32_t col_term[WN];
    float sw[WN];
#pragma unroll
    for (int bj = 0; bj < WN; ++bj) {
        col_term[bj] = base - 2u * ca * pw[bj];
        const int64_t n = n_lane + bj * 32;
        sw[bj] = (g.w_scale && n < g.N) ? half_bits_to_float(g.w_scale[n]) : 1.0f;
    }
    auto emit = [&](auto guard_c, auto i32_c, auto f16_c) __attribute__((always_inline)) {
        constexpr bool GUARD = decltype(guard_c)::value, I32 = decltype(i32_c)::value, F16 = decltype(f16_c)::value;
        int32_t *ci = I32 ? g.c_i32 + m_lane * g.N + n_lane : nullptr;
        uint16_t *ch = F16 ? g.c_f16 + m_lane * g.N + n_lane : nullptr;
#pragma unroll
        for (int bi = 0; bi < WM; ++bi) {
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int4 pa = pa4(bi, v4);
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
                        const uint32_t c = Acc<FP4>::four_s(acc[bi][bj][4 * v4 + r]) + row_term[r] + col_term[bj];
                        if constexpr (I32) ci[row * g.N + bj * 32] = (int32_t)c;
                        if constexpr (F16) ch[row * g.N + bj * 32] = float_to_half_bits((float)(int32_t)c * sa * sw[bj]);
                    }
                }
            }
        }
    };
    using T = std::true_type;
    using F = std::false_type;
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

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so that
// the packed rows it re-reads stay in its own L2.
__device__ __forceinline__ int xcd_tile_id(int block, int tiles_total)
{
    if ((tiles_total & 7) == 0) return (block & 7) * (tiles_total >> 3) + (block >> 3);
    return block;
}

}  // namespace mfma
}  // namespace apmm
