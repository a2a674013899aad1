// Pack / unpack kernels: paper Sec. 4.1 (matrix decomposition and reassembly).
//   step 1  split every code into its bits (planes)
//   step 2  reassemble each plane into 32-bit words
//   step 3  concatenate the planes (here: tile-interleaved, see apmm_layout.h)
// plus, behind the planes, one int32 per row: the sum of the row's codes over the padded K
// (= sum_i 2^i popcount(plane i)), which the MFMA kernels need for the recovery and which costs
// one popcount per packed word here instead of one per word and output tile there.
//
// One wave owns one row: lane l packs the 32-element groups l, l+64, ... (two 16-byte loads of
// codes, one word per plane out) and keeps a running code sum; the wave adds the 64 partial sums
// with lane shuffles.  No atomics, no LDS.  The work is HBM bound: 1 byte read and bits/8 bytes
// written per element.
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
    const int64_t groups = nkb * kWordsPerRow;  // 32-element groups per row
    uint32_t sum = 0;                           // sum_i 2^i popcount(plane i) over this lane's groups

    for (int64_t kg = lane; kg < groups; kg += 64) {
        // d[t4] = four consecutive codes 4*t4 .. 4*t4+3 of the group, one per byte
        uint32_t d[8];
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
        } else {
#pragma unroll
            for (int t4 = 0; t4 < 8; ++t4) d[t4] = 0u;
        }

        const int64_t kb = kg / kWordsPerRow;
        const int g = (int)(kg % kWordsPerRow);
        uint32_t *dst = packed + tile_row_word(row, kb, nkb, bits, 0) + g;
        for (int i = 0; i < bits; ++i) {
            uint32_t word = 0;
#pragma unroll
            for (int t4 = 0; t4 < 8; ++t4) word |= ((d[t4] >> i) & 0x01010101u) << t4;
            dst[i * kPlaneWords] = __builtin_rotateleft32(word, plane_rotation(i));
            sum += (uint32_t)__popc(word) << i;
        }
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
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= rows * groups) return;
    const int64_t row = t / groups;
    const int64_t kg = t % groups;
    const int64_t kb = kg / kWordsPerRow;
    const int g = (int)(kg % kWordsPerRow);
    const uint32_t *src = packed + tile_row_word(row, kb, nkb, bits, 0) + g;

    uint32_t d[8];
#pragma unroll
    for (int t4 = 0; t4 < 8; ++t4) d[t4] = 0u;
    for (int i = 0; i < bits; ++i) {
        const uint32_t word = __builtin_rotateright32(src[i * kPlaneWords], plane_rotation(i));
#pragma unroll
        for (int t4 = 0; t4 < 8; ++t4) d[t4] |= ((word >> t4) & 0x01010101u) << i;
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
