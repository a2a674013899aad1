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
// (they are small and stay in L1/L2).
#include "apmm_epilogue.h"
#include "apmm_kernels.h"

namespace apmm {
namespace {

constexpr int kTile = 16;

__global__ __launch_bounds__(kTile * kTile) void gemm_valu_kernel(GemmArgs g)
{
    const int64_t n = (int64_t)blockIdx.x * kTile + threadIdx.x;
    const int64_t m = (int64_t)blockIdx.y * kTile + threadIdx.y;
    if (m >= g.M || n >= g.N) return;
    const int p = g.p, q = g.q;

    uint32_t weighted = 0;  // sum_ij 2^(i+j) popcount, modulo 2^32 (the true C fits 32 bits)
    for (int64_t kb = 0; kb < g.nkb; ++kb) {
        const uint4 *arow = reinterpret_cast<const uint4 *>(g.a + tile_row_word(m, kb, g.nkb, p, 0));
        const uint4 *wrow = reinterpret_cast<const uint4 *>(g.w + tile_row_word(n, kb, g.nkb, q, 0));
        for (int i = 0; i < q; ++i) {
            const uint4 wv = wrow[i * (kPlaneWords / 4)];
            for (int j = 0; j < p; ++j) {
                // plane words are stored rotated by their plane index: bring the activation plane
                // to the weight plane's rotation before comparing
                const uint4 av = arow[j * (kPlaneWords / 4)];
                const int r = (plane_rotation(j) - plane_rotation(i)) & 31;
                const uint32_t pc = __popc(__builtin_rotateright32(av.x, r) ^ wv.x) +
                                    __popc(__builtin_rotateright32(av.y, r) ^ wv.y) +
                                    __popc(__builtin_rotateright32(av.z, r) ^ wv.z) +
                                    __popc(__builtin_rotateright32(av.w, r) ^ wv.w);
                weighted += pc << (i + j);
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
    if (gx > 0x7fffffffLL || gy > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_valu_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(kTile, kTile), 0, stream, args);
    return hipGetLastError();
}

}  // namespace apmm
