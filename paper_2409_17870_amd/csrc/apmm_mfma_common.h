// Pieces shared by the MFMA GEMM kernels: compile-time loops, the packed word -> operand expansion
// for the two operand formats, the workgroup -> tile map.
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
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), always flattened,
// so that every index below is a constant (shift amounts, register numbers).
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

template <int C>
__device__ __forceinline__ uint32_t vec_word(const uint4 &u)
{
    return C == 0 ? u.x : C == 1 ? u.y : C == 2 ? u.z : u.w;
}
// word S[W], W = 0..7, of a pair group whose two slots are held as u0 = S[0..3], u1 = S[4..7]
template <int W>
__device__ __forceinline__ uint32_t pair_word(const uint4 &u0, const uint4 &u1)
{
    return W < 4 ? vec_word<W & 3>(u0) : vec_word<W & 3>(u1);
}

// ---- E2M1 (fp4) operands: v_mfma_scale_f32_*_f8f6f4, 32 codes per lane and MFMA = 4 dwords of 8 nibbles ----
// Pair group: the nibble is 00uu, whose E2M1 value is u/2 (patterns 0..3 are 0, 0.5, 1, 1.5: linear).
// Dword D = 2 tp + tt of k step KS comes from S[2 KS + tp], field tt of every nibble.
template <int KS, int D>
__device__ __forceinline__ uint32_t fp4_pair_dword(const uint4 &u0, const uint4 &u1)
{
    const uint32_t w = pair_word<2 * KS + D / 2>(u0, u1);
    return (D & 1) ? (w >> 2) & 0x33333333u : w & 0x33333333u;
}
// Single group: the bit of k step KS stands at position KS of every nibble of L[D].  Positions 0, 1, 2
// are the E2M1 values 0.5, 1, 2 (position 3 is the sign: moved to position 2); the MFMA's power-of-two
// operand scale takes the factor 2^KS (resp. 4) out again: add fp4_single_exponent(KS) to the exponent.
template <int KS, int D>
__device__ __forceinline__ uint32_t fp4_single_dword(const uint4 &u)
{
    const uint32_t l = vec_word<D>(u);
    return KS < 3 ? l & (0x11111111u << KS) : (l >> 1) & 0x44444444u;
}
constexpr int fp4_single_exponent(int ks) { return ks < 3 ? -ks : -2; }

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so that
// the packed rows it re-reads stay in its own L2.
__device__ __forceinline__ int xcd_tile_id(int block, int tiles_total)
{
    if ((tiles_total & 7) == 0) return (block & 7) * (tiles_total >> 3) + (block >> 3);
    return block;
}

}  // namespace mfma
}  // namespace apmm
