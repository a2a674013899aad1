// Pack / unpack kernels: paper Sec. 4.1 (matrix decomposition and reassembly).
//   step 1  split every code into its bits (planes)
//   step 2  reassemble the planes into 32-bit words
//   step 3  concatenate them (here: tile-interleaved and grouped for the consumers, see apmm_layout.h)
// plus, behind the tiles, one int32 per row: the sum of the row's codes over the padded K, which the
// MFMA kernels need for the recovery and which costs one byte-sum per four codes here instead of
// popcounts per word and output tile there.
//
// One wave owns one row: lane l packs the 32-element groups l, l+64, ... (two 16-byte loads of
// codes) and keeps a running code sum; the wave adds the 64 partial sums with lane shuffles.  A pair
// group gives two whole words per lane; the words of a single group collect one bit position from
// each of the four 32-element groups of a k block, i.e. from four neighbouring lanes, which are
// OR-ed together with two lane exchanges.  No atomics, no LDS.  The work is HBM bound: 1 byte read
// and bits/8 bytes written per element.
#include <hip/hip_fp16.h>

#include "apmm_kernels.h"

namespace apmm {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerWg = kThreads / 64;

// Packs one 32-element group kg of a row: d[2t + jh] = the four codes 8t + 4jh + (0..3), one per byte,
// already masked to `bits` bits.  Adds the codes to `sum`.  The four lanes 4x .. 4x+3 of a wave must hold
// the four groups ks = 0..3 of one k block and call this together (single groups exchange words).
__device__ __forceinline__ void pack_group(uint32_t *__restrict__ packed, int64_t row, int64_t nkb, int bits,
                                           int64_t kg, const uint32_t (&d)[8], uint32_t &sum)
{
#pragma unroll
    for (int t4 = 0; t4 < 8; ++t4) sum = __builtin_amdgcn_sad_u8(d[t4], 0u, sum);  // + the four bytes
    const int64_t kb = kg / kWordsPerRow;
    const int ks = (int)(kg % kWordsPerRow);
    for (int h = 0; h < pair_groups(bits); ++h) {
        // S[2 ks + tp], tp = 0, 1: slot 2h + ks/2, words 2 (ks % 2) + tp
        uint32_t s[2];
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
            uint32_t word = 0;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int jh = 0; jh < 2; ++jh)
                    word |= ((d[2 * (2 * tp + tt) + jh] >> (2 * h)) & 0x03030303u) << (4 * jh + 2 * tt);
            s[tp] = word;
        }
        uint32_t *dst = packed + tile_row_word(row, kb, nkb, bits, 2 * h + (ks >> 1)) + 2 * (ks & 1);
        *reinterpret_cast<uint2 *>(dst) = make_uint2(s[0], s[1]);
    }
    if (has_single_group(bits)) {
        uint32_t l[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t word = 0;
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) word |= ((d[2 * t + jh] >> (bits - 1)) & 0x01010101u) << (4 * jh);
            word <<= ks;
            word |= __shfl_xor(word, 1);
            word |= __shfl_xor(word, 2);
            l[t] = word;
        }
        // every lane of the four now holds L[0..3]; lane ks stores L[ks]
        const uint32_t mine = ks == 0 ? l[0] : ks == 1 ? l[1] : ks == 2 ? l[2] : l[3];
        packed[tile_row_word(row, kb, nkb, bits, bits - 1) + ks] = mine;
    }
}

// The same for the field form of 3- and 4-bit activations (apmm_layout.h): the 32 codes of the group
// become the 192-bit E2M3 operand of k step ks, field 8 t + 2 c + jh at bit 6 (8 t + 2 c + jh).
__device__ __forceinline__ uint64_t spread_bytes_12(uint32_t x)
{
    // byte c of x -> bits 12 c .. 12 c + 7
    return (uint64_t)((x & 0xffu) | ((x & 0xff00u) << 4) | ((x & 0xff0000u) << 8)) | ((uint64_t)(x >> 24) << 36);
}

__device__ __forceinline__ void pack_group_fields(uint32_t *__restrict__ packed, int64_t row, int64_t nkb, int64_t kg,
                                                  const uint32_t (&d)[8], uint32_t &sum)
{
#pragma unroll
    for (int t4 = 0; t4 < 8; ++t4) sum = __builtin_amdgcn_sad_u8(d[t4], 0u, sum);
    const int64_t kb = kg / kWordsPerRow;
    const int ks = (int)(kg % kWordsPerRow);
    uint64_t chunk[4];  // the 48 bits of t = 0..3
#pragma unroll
    for (int t = 0; t < 4; ++t) chunk[t] = spread_bytes_12(d[2 * t]) | (spread_bytes_12(d[2 * t + 1]) << 6);
    const uint32_t dw0 = (uint32_t)chunk[0], dw1 = (uint32_t)(chunk[0] >> 32) | ((uint32_t)chunk[1] << 16),
                   dw2 = (uint32_t)(chunk[1] >> 16), dw3 = (uint32_t)chunk[2],
                   dw4 = (uint32_t)(chunk[2] >> 32) | ((uint32_t)chunk[3] << 16), dw5 = (uint32_t)(chunk[3] >> 16);
    // words 6 ks .. 6 ks + 5 of the row's 24: slot w / 4, word w % 4
    uint32_t *base = packed + tile_row_word(row, kb, nkb, 6, 0) + 3 * (ks >> 1) * kPlaneWords;
    if ((ks & 1) == 0) {
        *reinterpret_cast<uint4 *>(base) = make_uint4(dw0, dw1, dw2, dw3);
        *reinterpret_cast<uint2 *>(base + kPlaneWords) = make_uint2(dw4, dw5);
    } else {
        *reinterpret_cast<uint2 *>(base + kPlaneWords + 2) = make_uint2(dw0, dw1);
        *reinterpret_cast<uint4 *>(base + 2 * kPlaneWords) = make_uint4(dw2, dw3, dw4, dw5);
    }
}

__global__ __launch_bounds__(kThreads) void pack_kernel(const uint8_t *__restrict__ codes, int64_t rows,
                                                        int64_t K, int bits, uint32_t *__restrict__ packed,
                                                        int64_t rows_p, int64_t nkb, bool field)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 6);
    if (row >= rows_p) return;
    const int64_t groups = nkb * kWordsPerRow;  // 32-element groups per row, a multiple of 16
    const uint32_t code_mask = 0x01010101u * ((1u << bits) - 1u);
    uint32_t sum = 0;                           // sum of the codes of this lane's groups

    auto load_group = [&](int64_t kg, uint32_t (&d)[8]) __attribute__((always_inline)) {
        if (row < rows) {
            const int64_t k0 = kg * 32;
            const uint8_t *src = codes + row * K + k0;
            if (k0 + 32 <= K && (((uintptr_t)src) & 15) == 0) {
                const uint4 lo = *reinterpret_cast<const uint4 *>(src);
                const uint4 hi = *reinterpret_cast<const uint4 *>(src + 16);
                d[0] = lo.x; d[1] = lo.y; d[2] = lo.z; d[3] = lo.w;
                d[4] = hi.x; d[5] = hi.y; d[6] = hi.z; d[7] = hi.w;
            } else {
#pragma unroll
                for (int t4 = 0; t4 < 8; ++t4) {
                    uint32_t v = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int64_t k = k0 + 4 * t4 + c;
                        const uint32_t code = (k < K) ? src[4 * t4 + c] : 0xffu;  // pad: every plane bit set
                        v |= code << (8 * c);
                    }
                    d[t4] = v;
                }
            }
#pragma unroll
            for (int t4 = 0; t4 < 8; ++t4) d[t4] &= code_mask;
        } else {
#pragma unroll
            for (int t4 = 0; t4 < 8; ++t4) d[t4] = 0u;
        }
    };

    // two groups per lane and pass, both loaded before either is packed (more bytes in flight);
    // groups is a multiple of 16, so the lanes 4x .. 4x+3 always take the same branch
    for (int64_t kg = lane; kg < groups; kg += 128) {
        uint32_t d0[8], d1[8];
        const bool second = kg + 64 < groups;
        load_group(kg, d0);
        if (second) load_group(kg + 64, d1);
        if (field) {
            pack_group_fields(packed, row, nkb, kg, d0, sum);
            if (second) pack_group_fields(packed, row, nkb, kg + 64, d1, sum);
        } else {
            pack_group(packed, row, nkb, bits, kg, d0, sum);
            if (second) pack_group(packed, row, nkb, bits, kg + 64, d1, sum);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) packed[row_sum_word(rows_p, nkb, field ? 6 : bits) + row] = sum;
}

// Fused quantise + pack (paper Sec. 3.1: the feature matrix is quantised onto the symmetric bipolar-INT
// grid; Sec. 4.1: decomposition and reassembly).  One wave per row (token):
//   1. max |x| over the row (on the bit patterns, two halves per operation);
//      scale = half(max|x| / (2^bits - 1)), stored per token; r = 1 / scale;
//   2. u = clamp(floor(x * (r / 2)) + 2^(bits-1), 0, 2^bits - 1): x / scale moved to the nearest odd
//      integer (ties upward), as a code; then the same packing as pack_kernel.
// Rows of up to 8192 elements stay in registers between the two steps; longer rows are read again (from
// L2).  Single precision throughout, so that the codes are a function of the inputs alone.  A row whose
// scale rounds to zero gets the code of +1 everywhere.
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
constexpr int kCachedGroups = 4;  // 32-element groups per lane kept in registers

__global__ __launch_bounds__(kThreads) void quantize_pack_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                                 int64_t K, int bits,
                                                                 uint32_t *__restrict__ packed,
                                                                 uint16_t *__restrict__ scale_out, int64_t rows_p,
                                                                 int64_t nkb, bool field)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 6);
    if (row >= rows_p) return;
    const int64_t groups = nkb * kWordsPerRow;
    const uint16_t *xrow = x + row * K;
    const bool vec_ok = ((K & 7) == 0) && ((((uintptr_t)x) & 15) == 0);  // every group start is 16-byte aligned

    // h[i] = elements 2i, 2i+1 of group kg as two binary16 bit patterns; elements past K read as +0
    auto load_halves = [&](int64_t kg, uint32_t (&h)[16]) __attribute__((always_inline)) {
        const int64_t k0 = kg * 32;
        if (vec_ok && k0 + 32 <= K) {
            const uint4 *src = reinterpret_cast<const uint4 *>(xrow + k0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint4 q = src[v];
                h[4 * v] = q.x; h[4 * v + 1] = q.y; h[4 * v + 2] = q.z; h[4 * v + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t k = k0 + 2 * i;
                const uint32_t lo = k < K ? xrow[k] : 0u, hi = k + 1 < K ? xrow[k + 1] : 0u;
                h[i] = lo | (hi << 16);
            }
        }
    };
    auto fold_max = [](us2 m, const uint32_t (&h)[16]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t mag = h[i] & 0x7fff7fffu;  // |x| orders like its bit pattern
            m = __builtin_elementwise_max(m, us2{(unsigned short)(mag & 0xffffu), (unsigned short)(mag >> 16)});
        }
        return m;
    };

    const bool live = row < rows;
    const int64_t live_groups = live ? (K + 31) / 32 : 0;  // groups that hold at least one element
    uint32_t cache[kCachedGroups][16];
    us2 m2 = {0, 0};
#pragma unroll
    for (int it = 0; it < kCachedGroups; ++it) {
        const int64_t kg = lane + 64 * it;
        if (kg < live_groups) {
            load_halves(kg, cache[it]);
            m2 = fold_max(m2, cache[it]);
        }
    }
    for (int64_t kg = lane + 64 * kCachedGroups; kg < live_groups; kg += 64) {
        uint32_t h[16];
        load_halves(kg, h);
        m2 = fold_max(m2, h);
    }
    uint32_t mbits = m2[0] > m2[1] ? m2[0] : m2[1];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t o = __shfl_xor(mbits, off);
        mbits = o > mbits ? o : mbits;
    }
    const float amax = __half2float(__ushort_as_half((uint16_t)mbits));
    const uint32_t top = (1u << bits) - 1u;
    const __half sh = __float2half_rn(amax / (float)top);
    const float s = __half2float(sh);
    if (live && lane == 0) scale_out[row] = __half_as_ushort(sh);
    const float half_r = s > 0.0f ? (1.0f / s) * 0.5f : 0.0f;  // scale 0: every code becomes 2^(bits-1)
    const float mid = (float)(1u << (bits - 1)), ftop = (float)top;

    uint32_t sum = 0;
    // codes of group kg from its halves h (elements past K: the all-ones padding code), then the packing
    auto quantize_group = [&](int64_t kg, const uint32_t (&h)[16]) __attribute__((always_inline)) {
        uint32_t d[8];
        const bool whole = kg * 32 + 32 <= K;
#pragma unroll
        for (int t4 = 0; t4 < 8; ++t4) {
            uint32_t v = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t pair = h[2 * t4 + (c >> 1)];
                const float xf = __half2float(__ushort_as_half((uint16_t)((c & 1) ? pair >> 16 : pair & 0xffffu)));
                float u = floorf(xf * half_r) + mid;  // exact: |floor| is far below 2^24
                u = __builtin_amdgcn_fmed3f(u, 0.0f, ftop);
                if (!whole && kg * 32 + 4 * t4 + c >= K) u = ftop;
                v = __builtin_amdgcn_cvt_pk_u8_f32(u, c, v);  // byte c of v = u
            }
            d[t4] = v;
        }
        if (field) pack_group_fields(packed, row, nkb, kg, d, sum);
        else pack_group(packed, row, nkb, bits, kg, d, sum);
    };
    auto fill_group = [&](int64_t kg) __attribute__((always_inline)) {
        // a whole group of padding (every plane bit set) or a padding row (zero words)
        uint32_t d[8];
        const uint32_t fill = live ? 0x01010101u * top : 0u;
#pragma unroll
        for (int t4 = 0; t4 < 8; ++t4) d[t4] = fill;
        if (field) pack_group_fields(packed, row, nkb, kg, d, sum);
        else pack_group(packed, row, nkb, bits, kg, d, sum);
    };
    // The four lanes that pack a k block together must take the same call: a k block with any live group
    // quantises all four of its groups (elements past K become padding codes inside quantize_group).
    const int64_t live_blocks4 = (live_groups + 3) / 4 * 4;
#pragma unroll
    for (int it = 0; it < kCachedGroups; ++it) {
        const int64_t kg = lane + 64 * it;
        if (kg < live_blocks4) {
            if (kg >= live_groups) {
#pragma unroll
                for (int i = 0; i < 16; ++i) cache[it][i] = 0u;
            }
            quantize_group(kg, cache[it]);
        } else if (kg < groups) {
            fill_group(kg);
        }
    }
    for (int64_t kg = lane + 64 * kCachedGroups; kg < groups; kg += 64) {
        if (kg < live_blocks4) {
            uint32_t h[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) h[i] = 0u;
            if (kg < live_groups) load_halves(kg, h);
            quantize_group(kg, h);
        } else {
            fill_group(kg);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) packed[row_sum_word(rows_p, nkb, field ? 6 : bits) + row] = sum;
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint32_t *__restrict__ packed, int64_t rows,
                                                          int64_t K, int bits, uint8_t *__restrict__ codes,
                                                          int64_t nkb, bool field)
{
    const int64_t groups = nkb * kWordsPerRow;
    const int64_t th = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (th >= rows * groups) return;
    const int64_t row = th / groups;
    const int64_t kg = th % groups;
    const int64_t kb = kg / kWordsPerRow;
    const int ks = (int)(kg % kWordsPerRow);

    uint32_t d[8];
#pragma unroll
    for (int t4 = 0; t4 < 8; ++t4) d[t4] = 0u;
    if (field) {
        // words 6 ks .. 6 ks + 5 of the row's 24 hold the 32 six-bit fields of this group
        const uint32_t *base = packed + tile_row_word(row, kb, nkb, 6, 0);
        uint32_t dw[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int w = 6 * ks + i;
            dw[i] = base[(w >> 2) * kPlaneWords + (w & 3)];
        }
        const uint64_t chunk[4] = {(uint64_t)dw[0] | ((uint64_t)(dw[1] & 0xffffu) << 32),
                                   (uint64_t)(dw[1] >> 16) | ((uint64_t)dw[2] << 16),
                                   (uint64_t)dw[3] | ((uint64_t)(dw[4] & 0xffffu) << 32),
                                   (uint64_t)(dw[4] >> 16) | ((uint64_t)dw[5] << 16)};
        const uint32_t code_mask = (1u << bits) - 1u;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int jh = 0; jh < 2; ++jh)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    d[2 * t + jh] |= ((uint32_t)(chunk[t] >> (12 * c + 6 * jh)) & code_mask) << (8 * c);
    }
    for (int h = 0; !field && h < pair_groups(bits); ++h) {
        const uint32_t *src = packed + tile_row_word(row, kb, nkb, bits, 2 * h + (ks >> 1)) + 2 * (ks & 1);
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
            const uint32_t word = src[tp];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int jh = 0; jh < 2; ++jh)
                    d[2 * (2 * tp + tt) + jh] |= ((word >> (4 * jh + 2 * tt)) & 0x03030303u) << (2 * h);
        }
    }
    if (!field && has_single_group(bits)) {
        const uint32_t *src = packed + tile_row_word(row, kb, nkb, bits, bits - 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t word = src[t] >> ks;
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) d[2 * t + jh] |= ((word >> (4 * jh)) & 0x01010101u) << (bits - 1);
        }
    }
    const int64_t k0 = kg * 32;
    uint8_t *dst = codes + row * K + k0;
#pragma unroll
    for (int t4 = 0; t4 < 8; ++t4)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (k0 + 4 * t4 + c < K) dst[4 * t4 + c] = (uint8_t)(d[t4] >> (8 * c));
}

}  // namespace

hipError_t launch_pack(const uint8_t *codes, int64_t rows, int64_t K, int bits, bool field, uint32_t *packed,
                       hipStream_t stream)
{
    const int64_t rows_p = round_up(rows, kRowBlock);
    const int64_t nkb = round_up(K, kKPad) / kKBlock;
    if (rows_p == 0) return hipSuccess;
    const int64_t blocks = (rows_p + kRowsPerWg - 1) / kRowsPerWg;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, codes, rows, K, bits,
                       packed, rows_p, nkb, field);
    return hipGetLastError();
}

hipError_t launch_quantize_pack(const uint16_t *x, int64_t rows, int64_t K, int bits, bool field, uint32_t *packed,
                                uint16_t *scale, hipStream_t stream)
{
    const int64_t rows_p = round_up(rows, kRowBlock);
    const int64_t nkb = round_up(K, kKPad) / kKBlock;
    if (rows_p == 0) return hipSuccess;
    const int64_t blocks = (rows_p + kRowsPerWg - 1) / kRowsPerWg;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_pack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, rows, K, bits,
                       packed, scale, rows_p, nkb, field);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t *packed, int64_t rows, int64_t K, int bits, bool field, uint8_t *codes,
                         hipStream_t stream)
{
    const int64_t nkb = round_up(K, kKPad) / kKBlock;
    const int64_t total = rows * nkb * kWordsPerRow;
    if (total == 0) return hipSuccess;
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, packed, rows, K, bits,
                       codes, nkb, field);
    return hipGetLastError();
}

}  // namespace apmm
