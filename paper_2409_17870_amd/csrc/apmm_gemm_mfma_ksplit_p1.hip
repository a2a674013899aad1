// K-split MFMA GEMM kernels (apmm_gemm_mfma_ksplit.h) for 1-bit activations and 1..4-bit weights.
#include "apmm_gemm_mfma_ksplit.h"

namespace apmm {

namespace {
template <int Q>
hipError_t launch_q(const GemmArgs &g, hipStream_t stream, int wn)
{
    // activations in the group form: the 64 x 64 and 64 x 128 tiles (the wider ones measured slower)
    if (wn == 2) return mfma::launch_ksplit_variant<1, Q, 2, 2>(g, stream);
    return mfma::launch_ksplit_variant<1, Q, 2, 4>(g, stream);
}
}  // namespace

hipError_t launch_gemm_mfma_ksplit_p1(const GemmArgs &g, hipStream_t stream, int wn)
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
