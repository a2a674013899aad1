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
#include "apmm_kernels.h"

namespace apmm {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerWg = kThreads / 64;

__global__ __launch_bounds__(kThreads) void pack_kernel(const uint8_t *__restrict__ codes, int64_t rows,
                                                        int64_t K, int bits, uint32_t *__restrict__ packed,
                                                        int64_t rows_p, int64_t nkb)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 6);
    if (row >= rows_p) return;
    const int64_t groups = nkb * kWordsPerRow;  // 32-element groups per row, a multiple of 16
    const uint32_t code_mask = 0x01010101u * ((1u << bits) - 1u);
    uint32_t sum = 0;                           // sum of the codes of this lane's groups

    // d[2t + jh] = the four codes 8t + 4jh + (0..3) of group kg, one per byte (masked to `bits` bits)
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
    // the four lanes 4x .. 4x+3 hold the four groups ks = 0..3 of one k block
    auto pack_group = [&](int64_t kg, const uint32_t (&d)[8]) __attribute__((always_inline)) {
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
                for (int jh = 0; jh < 2; ++jh)
                    word |= ((d[2 * t + jh] >> (bits - 1)) & 0x01010101u) << (4 * jh);
                word <<= ks;
                word |= __shfl_xor(word, 1);
                word |= __shfl_xor(word, 2);
                l[t] = word;
            }
            // every lane of the four now holds L[0..3]; lane ks stores L[ks]
            const uint32_t mine = ks == 0 ? l[0] : ks == 1 ? l[1] : ks == 2 ? l[2] : l[3];
            packed[tile_row_word(row, kb, nkb, bits, bits - 1) + ks] = mine;
        }
    };

    // two groups per lane and pass, both loaded before either is packed (more bytes in flight);
    // groups is a multiple of 16, so the lanes 4x .. 4x+3 always take the same branch
    for (int64_t kg = lane; kg < groups; kg += 128) {
        uint32_t d0[8], d1[8];
        const bool second = kg + 64 < groups;
        load_group(kg, d0);
        if (second) load_group(kg + 64, d1);
        pack_group(kg, d0);
        if (second) pack_group(kg + 64, d1);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) packed[row_sum_word(rows_p, nkb, bits) + row] = sum;
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint32_t *__restrict__ packed, int64_t rows,
                                                          int64_t K, int bits, uint8_t *__restrict__ codes,
                                                          int64_t nkb)
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
    for (int h = 0; h < pair_groups(bits); ++h) {
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
    if (has_single_group(bits)) {
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

hipError_t launch_pack(const uint8_t *codes, int64_t rows, int64_t K, int bits, uint32_t *packed,
                       hipStream_t stream)
{
    const int64_t rows_p = round_up(rows, kRowBlock);
    const int64_t nkb = round_up(K, kKPad) / kKBlock;
    if (rows_p == 0) return hipSuccess;
    const int64_t blocks = (rows_p + kRowsPerWg - 1) / kRowsPerWg;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, codes, rows, K, bits,
                       packed, rows_p, nkb);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t *packed, int64_t rows, int64_t K, int bits, uint8_t *codes,
                         hipStream_t stream)
{
    const int64_t nkb = round_up(K, kKPad) / kKBlock;
    const int64_t total = rows * nkb * kWordsPerRow;
    if (total == 0) return hipSuccess;
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, packed, rows, K, bits,
                       codes, nkb);
    return hipGetLastError();
}

}  // namespace apmm
