// Packed bit-plane layout shared by every kernel of the library (paper Sec. 4.1).
//
// A rows x K operand of n-bit codes is stored with n bits per element in 32-bit words, concatenated
// tile by tile:
//
//   word(rb, kb, s, r, g)   rb = row / 32       row block (rows padded to a multiple of 32)
//                           kb = k / 128        k block   (K padded to a multiple of 512: nkb is a multiple of 4)
//                           s  = plane slot, 0 .. n-1 (16 bytes per row and slot)
//                           r  = row % 32
//                           g  = word inside the slot, 0 .. 3
//   index = (((rb * nkb + kb) * n + s) * 32 + r) * 4 + g
//
// so one (rb, kb) tile is 512*n contiguous bytes and inside a slot the 32 rows are 16 bytes each:
// when the lanes of a wave take one row each, every 16-byte load instruction reads one contiguous
// 512-byte run per row block.
//
// Which bit of which word holds plane i of element k is chosen for the consumers, the matrix-unit
// kernels first.  The planes of a code are taken in groups: bits (0,1), (2,3), ... form PAIR groups,
// and when n is odd the top bit is a SINGLE group.  With the element's position inside its k block
// written as
//       k % 128 = 32*ks + 8*t + 4*jh + c,   ks, t in 0..3, jh in 0..1, c in 0..3,   t = 2*tp + tt,
//   pair group h (code bits 2h, 2h+1) fills slots 2h and 2h+1, seen as eight words S[0..7]
//       (slot 2h + w/4, word w % 4):  bit b of the group sits in S[2*ks + tp] at bit 8*c + 4*jh + 2*tt + b;
//   a single group (code bit n-1) fills slot n-1, four words L[0..3]:
//       the bit sits in L[t] at bit 8*c + 4*jh + ks.
// Reading them (apmm_mfma_common.h has the code):
//   * E2M1 (fp4) MFMA operand of k step ks: its four dwords are (S[2ks + tp] >> 2tt) & 0x33333333, i.e.
//     every nibble is 00uu with the 2-bit code of the group: 1.5 operations per dword.  For a single
//     group L[t] & (0x11111111 << ks): the bit stands at another place of the nibble in every k step,
//     which the MFMA's power-of-two operand scale undoes (1.25 operations per dword).
//   * XOR/popcount: (S[w] >> b) & 0x55555555 is plane 2h+b of 16 elements; two single-group words give
//     the same 16 elements with two shift-and-mask steps, so any two planes can be compared.
// Both operands of a GEMM use the same element -> (ks, t, jh, c) map, which is all a contraction needs.
//
// Activations of 3 or 4 bits use a second form, the FIELD form: six slots per (row, k block), i.e. 24
// words, six per k step ks (words 6 ks .. 6 ks + 5 of the row's 24, slot w / 4, word w % 4).  The 192 bits
// of a k step hold its 32 codes as 6-bit fields, field 8 t + 2 c + jh at bits 6 (8 t + 2 c + jh) ..., code in
// the low bits: exactly the E2M3 (fp6) MFMA operand of that k step, in which a 4-bit code u is the number
// u / 8.  The matrix unit multiplies fp6 and fp4 operands at the same rate, so 4-bit activations need no
// second sweep of K and no expansion at all, at the price of 6 instead of 4 bits per element in a buffer
// that lives for one GEMM (weights always keep the compact group form).
//
// Behind the tiles follows one int32 per (padded) row: the sum of the row's codes over the padded K.
// The MFMA kernels multiply codes u instead of values 2u - (2^n - 1) and need these sums to recover C.
//
// Padding: elements with k >= K have every plane bit set in BOTH operands.  Their XOR is zero, and each
// contributes exactly (2^p - 1)(2^q - 1) to an integer dot product, which the kernels subtract again.
// Rows >= `rows` are all-zero words and are never stored to C.
#pragma once
#include <stdint.h>

namespace apmm {

constexpr int kRowBlock = 32;    // rows per packed tile
constexpr int kKBlock = 128;     // k elements per packed tile
constexpr int kKPad = 512;       // K is padded to a multiple of this (four k blocks = two stages of the MFMA kernel)
constexpr int kWordsPerRow = 4;  // 32-bit words per (row, slot) inside a tile
constexpr int kPlaneWords = kRowBlock * kWordsPerRow;  // words between consecutive slots of a tile

inline __host__ __device__ int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// number of pair groups of an n-bit code, and whether a single group follows them
inline __host__ __device__ constexpr int pair_groups(int n) { return n / 2; }
inline __host__ __device__ constexpr bool has_single_group(int n) { return (n & 1) != 0; }

// activations of 3 or 4 bits are stored in the field form (six slots), everything else in the group form
inline __host__ __device__ constexpr bool activation_field_form(int p) { return p == 3 || p == 4; }
inline __host__ __device__ constexpr int activation_slots(int p) { return activation_field_form(p) ? 6 : p; }

// index of word g=0 of (row, slot s) in k block kb
inline __host__ __device__ int64_t tile_row_word(int64_t row, int64_t kb, int64_t nkb, int n, int s)
{
    int64_t rb = row / kRowBlock, r = row % kRowBlock;
    return (((rb * nkb + kb) * n + s) * kRowBlock + r) * kWordsPerRow;
}

// index of the first row-sum word: the tiles of rows_p x nkb*128 elements come first
inline __host__ __device__ int64_t row_sum_word(int64_t rows_p, int64_t nkb, int n)
{
    return rows_p * nkb * n * (kKBlock / 32);
}

struct GemmArgs {
    int64_t M, N, K;
    int64_t nkb;          // roundup(K,512)/128
    int p, q;
    const uint32_t *a;    // packed activations (null when a_codes is given)
    const uint8_t *a_codes;  // small-M kernels only: M x K activation codes, packed by the kernel itself; else null
    const uint32_t *w;    // packed weights
    const int32_t *a_sum; // per activation row: sum of its codes over the padded K
    const int32_t *w_sum; // per weight row: the same
    int32_t *c_i32;       // may be null
    uint16_t *c_f16;      // may be null
    const uint16_t *w_scale;  // may be null
    const uint16_t *a_scale;  // may be null
};

// Several problems of one launch (decode kernels): workgroups wg_end[i-1] .. wg_end[i]-1 work on g[i].
constexpr int kMaxGroup = 8;
struct GroupArgs {
    int count;
    int chunk_kb[kMaxGroup];  // per problem: k blocks of activations held on chip at a time (a multiple of 32, or all)
    int wg_end[kMaxGroup];
    GemmArgs g[kMaxGroup];
};

}  // namespace apmm
