// FP4 (E2M1) MFMA GEMM kernels for 1- and 2-bit operands; see apmm_gemm_mfma_impl.h.
#include "apmm_gemm_mfma_impl.h"

namespace apmm {
hipError_t launch_gemm_mfma_fp4_impl(const GemmArgs &g, hipStream_t stream) { return mfma::launch_fp4(g, stream); }
}  // namespace apmm
