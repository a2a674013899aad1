// Dispatch of the int8 MFMA GEMM (design A) over the activation width; the kernels are
// instantiated in apmm_gemm_mfma_p<P>.hip so that they compile in parallel.
#include "apmm_kernels.h"

namespace apmm {

hipError_t launch_gemm_mfma_p1(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p2(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p3(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p4(const GemmArgs &g, hipStream_t stream);

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
