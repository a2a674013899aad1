// Output stage shared by the GEMM kernels: the recovered int32 value is stored as is
// (the 32-bit output of paper Sec. 3.2) and/or scaled per token and per output channel
// in fp32 and rounded once to binary16.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include "apmm_layout.h"

namespace apmm {

__device__ __forceinline__ float half_bits_to_float(uint16_t bits)
{
    return __half2float(__ushort_as_half(bits));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float x)
{
    return __half_as_ushort(__float2half_rn(x));
}

// scale for row m / column n (1.0f when the vector is absent)
__device__ __forceinline__ float load_scale(const uint16_t *scale, int64_t idx)
{
    return scale ? half_bits_to_float(scale[idx]) : 1.0f;
}

// The same as raw binary16 bits, for kernels that request the scale long before they need it: the conversion
// is a use of the loaded value, and a use is where the wave waits for the load.
__device__ __forceinline__ uint32_t load_scale_bits(const uint16_t *scale, int64_t idx)
{
    return scale ? (uint32_t)scale[idx] : 0x3c00u;  // 1.0
}

// Pins the first use of a value loaded early to this point of the program: without it the compiler moves pure
// arithmetic on the value (a conversion, a multiply) up to the load, and the wave waits there for the load, and
// for every load issued before it.
__device__ __forceinline__ uint32_t use_here(uint32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}

__device__ __forceinline__ void store_output(const GemmArgs &g, int64_t m, int64_t n, int32_t c, float sa,
                                             float sw)
{
    const int64_t o = m * g.N + n;
    if (g.c_i32) g.c_i32[o] = c;
    if (g.c_f16) g.c_f16[o] = float_to_half_bits((float)c * sa * sw);
}

}  // namespace apmm
