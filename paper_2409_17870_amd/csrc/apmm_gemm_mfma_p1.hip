// int8 MFMA GEMM kernels for 1-bit activations (all weight widths); see apmm_gemm_mfma_impl.h.
#include "apmm_gemm_mfma_impl.h"

namespace apmm {
hipError_t launch_gemm_mfma_p1(const GemmArgs &g, hipStream_t stream) { return mfma::launch_int8_p<1>(g, stream); }
}  // namespace apmm
