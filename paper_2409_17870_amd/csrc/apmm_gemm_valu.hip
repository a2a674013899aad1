// Design B: bit-plane GEMM on the vector ALU (paper Sec. 3.2 with the XOR form of the
// 1-bit product).  For planes a^(j) of the activations and w^(i) of the weights,
//   D_ij = K - 2 * popcount(a^(j) xor w^(i))        (bit 1 = +1, bit 0 = -1)
//   C    = sum_i sum_j 2^(i+j) * D_ij
//        = K * (2^p - 1)(2^q - 1) - 2 * sum_ij 2^(i+j) * popcount(a^(j) xor w^(i)).
// Padded k positions carry identical bits in both operands, so they add nothing to the
// popcounts and the true K appears in the constant.  The recovery (shift and add) is done
// in registers; nothing but C touches global memory.
//
// This kernel is the general one: any p, q in 1..8, any M, N, K.  It is the fallback for codes the
// matrix-unit kernels do not cover and the reference for design B at large M.  A workgroup of 256 threads
// owns 64 x 64 outputs, a thread 4 x 4 of them (rows ty + 16 i, columns tx + 16 j).  Per k block the
// workgroup brings every plane of its 64 + 64 rows to the same form, 16 elements per word at the even bit
// positions (apmm_layout.h), once, into LDS; then any activation plane can be XOR-ed with any weight plane:
// per output, plane pair and word one XOR, one popcount and one shift-and-add.  The vector ALU bounds it:
// 3 p q operations per output and 16 elements, i.e. about 0.2 effective POP/s for W1A2 if every issue slot
// of the chip did nothing else.
#include "apmm_epilogue.h"
#include "apmm_kernels.h"

namespace apmm {
namespace {

constexpr int kTile = 16;

// Plane i of the 16 elements (ks = w / 2, tp = w % 2, all tt, jh, c) of one row and k block, at bits
// 8c + 4jh + 2tt.  `tile_row` points at word 0 of (row, slot 0).
__device__ __forceinline__ uint32_t plane_half_word(const uint32_t *tile_row, int n, int i, int w)
{
    if (i < 2 * pair_groups(n)) {
        const uint32_t s = tile_row[(i / 2 * 2 + (w >> 2)) * kPlaneWords + (w & 3)];  // S[w] of pair group i / 2
        return (s >> (i & 1)) & 0x55555555u;
    }
    const uint32_t *l = tile_row + (n - 1) * kPlaneWords + 2 * (w & 1);  // L[2 tp], L[2 tp + 1]
    const int ks = w >> 1;
    return ((l[0] >> ks) & 0x11111111u) | (((l[1] >> ks) & 0x11111111u) << 2);
}

// The same from activations in the field form (3 and 4 bits): bit i of field 8 t + 2 c + jh of k step ks is
// bit 6 (8 t + 2 c + jh) + i of the 192 bits in words 6 ks .. 6 ks + 5 of the row's 24.
__device__ __forceinline__ uint32_t field_plane_half_word(const uint32_t *tile_row, int i, int w)
{
    const int ks = w >> 1, tp = w & 1;
    uint32_t out = 0;
    for (int tt = 0; tt < 2; ++tt)
        for (int jh = 0; jh < 2; ++jh)
            for (int c = 0; c < 4; ++c) {
                const int bit = 6 * (8 * (2 * tp + tt) + 2 * c + jh) + i;
                const int word = 6 * ks + (bit >> 5);
                const uint32_t v = tile_row[(word >> 2) * kPlaneWords + (word & 3)];
                out |= ((v >> (bit & 31)) & 1u) << (8 * c + 4 * jh + 2 * tt);
            }
    return out;
}

constexpr int kOutTile = 64;                 // outputs per workgroup and dimension
constexpr int kPerThread = kOutTile / kTile;  // outputs per thread and dimension

__global__ __launch_bounds__(kTile * kTile) void gemm_valu_kernel(GemmArgs g, int64_t tiles_n)
{
    // one-dimensional grid (the y dimension would cap M at about four million rows)
    const int64_t n0 = ((int64_t)blockIdx.x % tiles_n) * kOutTile, m0 = ((int64_t)blockIdx.x / tiles_n) * kOutTile;
    const int tid = threadIdx.x, tx = tid % kTile, ty = tid / kTile;
    const int p = g.p, q = g.q;
    const int64_t rows_a = round_up(g.M, kRowBlock), rows_b = round_up(g.N, kRowBlock);
    // plane words of one k block: [plane][word 0..7][row 0..63]; consecutive lanes read consecutive rows
    __shared__ uint32_t a_lds[8 * 8 * kOutTile], w_lds[8 * 8 * kOutTile];

    uint32_t weighted[kPerThread][kPerThread];  // sum_ij 2^(i+j) popcount, modulo 2^32 (the true C fits 32 bits)
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) weighted[i][j] = 0;

    for (int64_t kb = 0; kb < g.nkb; ++kb) {
        if (kb) __syncthreads();  // every thread is done with the previous k block
        // fill: one word of one plane of one row per job; rows past the operand read its last padded row
        for (int job = tid; job < (p + q) * 8 * kOutTile; job += kTile * kTile) {
            const int r = job % kOutTile, w = (job / kOutTile) % 8, plane = job / (8 * kOutTile);
            if (plane < p) {
                int64_t row = m0 + r;
                if (row >= rows_a) row = rows_a - 1;
                const uint32_t *arow = g.a + tile_row_word(row, kb, g.nkb, activation_slots(p), 0);
                a_lds[(plane * 8 + w) * kOutTile + r] =
                    activation_field_form(p) ? field_plane_half_word(arow, plane, w) : plane_half_word(arow, p, plane, w);
            } else {
                int64_t row = n0 + r;
                if (row >= rows_b) row = rows_b - 1;
                const uint32_t *wrow = g.w + tile_row_word(row, kb, g.nkb, q, 0);
                w_lds[((plane - p) * 8 + w) * kOutTile + r] = plane_half_word(wrow, q, plane - p, w);
            }
        }
        __syncthreads();
        for (int w = 0; w < 8; ++w) {
            for (int j = 0; j < p; ++j) {
                uint32_t av[kPerThread];
#pragma unroll
                for (int i = 0; i < kPerThread; ++i) av[i] = a_lds[(j * 8 + w) * kOutTile + ty + kTile * i];
                for (int i = 0; i < q; ++i) {
#pragma unroll
                    for (int jn = 0; jn < kPerThread; ++jn) {
                        const uint32_t wv = w_lds[(i * 8 + w) * kOutTile + tx + kTile * jn];
#pragma unroll
                        for (int im = 0; im < kPerThread; ++im)
                            weighted[im][jn] += (uint32_t)__popc(av[im] ^ wv) << (i + j);
                    }
                }
            }
        }
    }
    const uint32_t full = (uint32_t)g.K * (uint32_t)((1 << p) - 1) * (uint32_t)((1 << q) - 1);
#pragma unroll
    for (int im = 0; im < kPerThread; ++im) {
        const int64_t m = m0 + ty + kTile * im;
        if (m >= g.M) continue;
        const float sa = load_scale(g.a_scale, m);
#pragma unroll
        for (int jn = 0; jn < kPerThread; ++jn) {
            const int64_t n = n0 + tx + kTile * jn;
            if (n < g.N) store_output(g, m, n, (int32_t)(full - 2u * weighted[im][jn]), sa, load_scale(g.w_scale, n));
        }
    }
}

}  // namespace

hipError_t launch_gemm_valu(const GemmArgs &args, hipStream_t stream)
{
    const int64_t gx = (args.N + kOutTile - 1) / kOutTile, gy = (args.M + kOutTile - 1) / kOutTile;
    if (gx > 0x7fffffffLL / gy) return hipErrorInvalidValue;
    note_kernel("gemm_valu_kernel");
    hipLaunchKernelGGL(gemm_valu_kernel, dim3((unsigned)(gx * gy)), dim3(kTile * kTile), 0, stream, args, gx);
    return hipGetLastError();
}

}  // namespace apmm
