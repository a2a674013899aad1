// E2M1 MFMA GEMM kernels for 1-bit activations and 1..4-bit weights.
#include "apmm_gemm_mfma_tiles.h"

namespace apmm {
hipError_t launch_gemm_mfma_fp4_p1(const GemmArgs &g, hipStream_t stream) { return mfma::launch_fp4_p<1>(g, stream); }
}  // namespace apmm
