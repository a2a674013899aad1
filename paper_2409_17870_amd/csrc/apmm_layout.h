// Packed bit-plane layout shared by every kernel of the library (paper Sec. 4.1).
//
// A rows x K operand of n-bit codes is stored as n one-bit planes in 32-bit words,
// concatenated tile by tile:
//
//   word(rb, kb, i, r, g)   rb = row / 32       row block (rows padded to a multiple of 32)
//                           kb = k / 128        k block   (K padded to a multiple of 512: nkb is a multiple of 4)
//                           i  = plane (bit of the code), 0 .. n-1
//                           r  = row % 32
//                           g  = (k % 128) / 32 word inside the k block
//   index = (((rb * nkb + kb) * n + i) * 32 + r) * 4 + g
//
// so one (rb, kb) tile is 512*n contiguous bytes, planes concatenated, and inside a plane the
// 32 rows are 16 bytes each: when the lanes of a wave take one row each, every 16-byte load
// instruction reads one contiguous 512-byte run per row block.
//
// Inside a word, element e = k % 32 of plane i sits at bit (8*(e % 4) + (e / 4) + i) mod 32:
// the "natural" word, whose byte c holds elements c, c+4, c+8, ..., rotated left by i.
// Masking plane i with 0x01010101 << ((t + i) % 8) keeps the bits of the four elements
// 4t .. 4t+3; OR-ing the masked planes and rotating right by t leaves, in each of the four
// bytes, bit i = plane bit i, i.e. the code u of the element as a byte.  That is the whole
// expansion to int8 MFMA operands: one AND(-OR) per plane and one rotate per four elements.
// XOR/popcount kernels rotate a plane word by the difference of the plane indices to compare
// planes of different index.
//
// Behind the planes of all tiles follows one int32 per (padded) row: the sum of the row's codes over
// the padded K, i.e. sum_i 2^i popcount(plane i).  The MFMA kernels multiply codes u instead of values
// 2u - (2^n - 1) and need these sums to recover C.
//
// Padding: elements with k >= K have every plane bit set in BOTH operands.  Their
// XOR is zero, and each contributes exactly (2^p - 1)(2^q - 1) to an integer dot
// product, which the kernels subtract again.  Rows >= `rows` are all-zero words and
// are never stored to C.
#pragma once
#include <stdint.h>

namespace apmm {

constexpr int kRowBlock = 32;    // rows per packed tile
constexpr int kKBlock = 128;     // k elements per packed tile
constexpr int kKPad = 512;       // K is padded to a multiple of this (four k blocks = two stages of the direct MFMA kernel)
constexpr int kWordsPerRow = 4;  // 32-bit words per (row, plane) inside a tile
constexpr int kPlaneWords = kRowBlock * kWordsPerRow;  // words between consecutive planes of a tile

// left rotation applied to the natural word of plane i
inline __host__ __device__ int plane_rotation(int i) { return i; }

inline __host__ __device__ int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// index of word g=0 of (row, plane i) in k block kb
inline __host__ __device__ int64_t tile_row_word(int64_t row, int64_t kb, int64_t nkb, int n, int i)
{
    int64_t rb = row / kRowBlock, r = row % kRowBlock;
    return (((rb * nkb + kb) * n + i) * kRowBlock + r) * kWordsPerRow;
}

// index of the first row-sum word: the planes of rows_p x nkb*128 elements come first
inline __host__ __device__ int64_t row_sum_word(int64_t rows_p, int64_t nkb, int n)
{
    return rows_p * nkb * n * (kKBlock / 32);
}

struct GemmArgs {
    int64_t M, N, K;
    int64_t nkb;          // roundup(K,128)/128
    int p, q;
    const uint32_t *a;    // packed activations
    const uint32_t *w;    // packed weights
    const int32_t *a_sum; // per activation row: sum of its codes over the padded K
    const int32_t *w_sum; // per weight row: the same
    int32_t *c_i32;       // may be null
    uint16_t *c_f16;      // may be null
    const uint16_t *w_scale;  // may be null
    const uint16_t *a_scale;  // may be null
    int32_t pad_corr;     // (Kp - K) * (2^p - 1) * (2^q - 1)
};

}  // namespace apmm
