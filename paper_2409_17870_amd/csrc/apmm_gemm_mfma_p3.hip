// int8 MFMA GEMM kernels for 3-bit activations (all weight widths); see apmm_gemm_mfma_impl.h.
#include "apmm_gemm_mfma_impl.h"

namespace apmm {
hipError_t launch_gemm_mfma_p3(const GemmArgs &g, hipStream_t stream) { return mfma::launch_int8_p<3>(g, stream); }
}  // namespace apmm
