// Dispatch of the int8 MFMA GEMM (design A) over the activation width; the kernels are
// instantiated in apmm_gemm_mfma_p<P>.hip so that they compile in parallel.
#include "apmm_kernels.h"

namespace apmm {

hipError_t launch_gemm_mfma_p1(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p2(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p3(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p4(const GemmArgs &g, hipStream_t stream);

// p, q in 1..4 are instantiated.  The raw MFMA sum S = sum ua * uw is bounded by the same
// K' (2^p - 1)(2^q - 1) <= INT32_MAX that the ABI checks, so no further limit applies.
bool gemm_mfma_supported(const GemmArgs &g) { return g.p >= 1 && g.p <= 4 && g.q >= 1 && g.q <= 4; }

hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t stream)
{
    switch (g.p) {
    case 1: return launch_gemm_mfma_p1(g, stream);
    case 2: return launch_gemm_mfma_p2(g, stream);
    case 3: return launch_gemm_mfma_p3(g, stream);
    case 4: return launch_gemm_mfma_p4(g, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace apmm
