// Design B: bit-plane GEMM on the vector ALU (paper Sec. 3.2 with the XOR form of the
// 1-bit product).  For planes a^(j) of the activations and w^(i) of the weights,
//   D_ij = K - 2 * popcount(a^(j) xor w^(i))        (bit 1 = +1, bit 0 = -1)
//   C    = sum_i sum_j 2^(i+j) * D_ij
//        = K * (2^p - 1)(2^q - 1) - 2 * sum_ij 2^(i+j) * popcount(a^(j) xor w^(i)).
// Padded k positions carry identical bits in both operands, so they add nothing to the
// popcounts and the true K appears in the constant.  The recovery (shift and add) is done
// in registers; nothing but C touches global memory.
//
// This kernel is the general one: any p, q in 1..8, any M, N, K.  One thread per output
// element, 16 x 16 outputs per workgroup; operands come straight from the packed tiles
// (they are small and stay in L1/L2).  It is the fallback for codes the matrix-unit kernels do
// not cover, written for clarity: every plane is brought to the same form, 16 elements per word
// at the even bit positions (apmm_layout.h), and then any activation plane can be XOR-ed with any
// weight plane.
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

__global__ __launch_bounds__(kTile * kTile) void gemm_valu_kernel(GemmArgs g, int64_t tiles_n)
{
    // one-dimensional grid (the y dimension would cap M at about a million rows)
    const int64_t n = ((int64_t)blockIdx.x % tiles_n) * kTile + threadIdx.x;
    const int64_t m = ((int64_t)blockIdx.x / tiles_n) * kTile + threadIdx.y;
    if (m >= g.M || n >= g.N) return;
    const int p = g.p, q = g.q;

    uint32_t weighted = 0;  // sum_ij 2^(i+j) popcount, modulo 2^32 (the true C fits 32 bits)
    for (int64_t kb = 0; kb < g.nkb; ++kb) {
        const uint32_t *arow = g.a + tile_row_word(m, kb, g.nkb, activation_slots(p), 0);
        const uint32_t *wrow = g.w + tile_row_word(n, kb, g.nkb, q, 0);
        for (int w = 0; w < 8; ++w) {
            uint32_t wp[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) wp[i] = i < q ? plane_half_word(wrow, q, i, w) : 0u;
            for (int j = 0; j < p; ++j) {
                const uint32_t ap = activation_field_form(p) ? field_plane_half_word(arow, j, w)
                                                              : plane_half_word(arow, p, j, w);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (i < q) weighted += (uint32_t)__popc(ap ^ wp[i]) << (i + j);
            }
        }
    }
    const uint32_t full = (uint32_t)g.K * (uint32_t)((1 << p) - 1) * (uint32_t)((1 << q) - 1);
    const int32_t c = (int32_t)(full - 2u * weighted);
    store_output(g, m, n, c, load_scale(g.a_scale, m), load_scale(g.w_scale, n));
}

}  // namespace

hipError_t launch_gemm_valu(const GemmArgs &args, hipStream_t stream)
{
    const int64_t gx = (args.N + kTile - 1) / kTile, gy = (args.M + kTile - 1) / kTile;
    if (gx > 0x7fffffffLL / gy) return hipErrorInvalidValue;
    note_kernel("gemm_valu_kernel");
    hipLaunchKernelGGL(gemm_valu_kernel, dim3((unsigned)(gx * gy)), dim3(kTile, kTile), 0, stream, args, gx);
    return hipGetLastError();
}

}  // namespace apmm
