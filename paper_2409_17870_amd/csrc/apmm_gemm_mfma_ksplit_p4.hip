// K-split MFMA GEMM kernels (apmm_gemm_mfma_ksplit.h) for 4-bit activations and 1..4-bit weights.
#include "apmm_gemm_mfma_ksplit.h"

namespace apmm {

namespace {
template <int Q>
hipError_t launch_q(const GemmArgs &g, hipStream_t stream, int wn)
{
    switch (wn) {
    case 2: return mfma::launch_ksplit_variant<4, Q, 2, 2>(g, stream);
    case 4: return mfma::launch_ksplit_variant<4, Q, 2, 4>(g, stream);
    case 5: return mfma::launch_ksplit_variant<4, Q, 2, 5>(g, stream);
    default: return mfma::launch_ksplit_variant<4, Q, 2, 6>(g, stream);
    }
}
}  // namespace

hipError_t launch_gemm_mfma_ksplit_p4(const GemmArgs &g, hipStream_t stream, int wn)
{
    switch (g.q) {
    case 1: return launch_q<1>(g, stream, wn);
    case 2: return launch_q<2>(g, stream, wn);
    case 3: return launch_q<3>(g, stream, wn);
    case 4: return launch_q<4>(g, stream, wn);
    }
    return hipErrorInvalidValue;
}

}  // namespace apmm
