// Dispatch of the MFMA GEMMs (design A).  The kernels are instantiated in
// apmm_gemm_mfma_p<P>.hip (int8 operands) and apmm_gemm_mfma_fp4.hip (E2M1 operands) so that
// they compile in parallel.
#include "apmm_kernels.h"

namespace apmm {

hipError_t launch_gemm_mfma_p1(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p2(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p3(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_p4(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_fp4_impl(const GemmArgs &g, hipStream_t stream);

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

// E2M1 holds the codes 0..3 exactly (as 0, 0.5, 1, 1.5); the fp32 accumulator holds S/4 in quarter
// units, exactly while S < 2^24: S <= 45 K' (4-bit x 2-bit codes), so K' up to 2^18 is safe; larger
// K goes to the int8 kernel.
bool gemm_mfma_fp4_supported(const GemmArgs &g)
{
    const bool p_ok = g.p == 1 || g.p == 2 || g.p == 4;  // 4-bit activations: two 2-bit plane groups
    return p_ok && g.q >= 1 && g.q <= 2 && g.nkb * kKBlock <= (1 << 18);
}

hipError_t launch_gemm_mfma_fp4(const GemmArgs &g, hipStream_t stream) { return launch_gemm_mfma_fp4_impl(g, stream); }

}  // namespace apmm
