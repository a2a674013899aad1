// Dispatch of the MFMA GEMMs (design A).  The kernels are instantiated in apmm_gemm_mfma_p<P>.hip,
// one translation unit per activation width, so that they compile in parallel.
#include <cstdarg>
#include <cstdio>

#include "apmm_kernels.h"

namespace apmm {

namespace {
thread_local KernelTiming g_timing = {nullptr, nullptr};
thread_local char g_last_kernel[96] = "";
}
void note_kernel(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_last_kernel, sizeof(g_last_kernel), fmt, ap);
    va_end(ap);
}
const char *last_kernel() { return g_last_kernel; }
void set_kernel_timing(hipEvent_t start, hipEvent_t stop) { g_timing = KernelTiming{start, stop}; }
KernelTiming take_kernel_timing()
{
    const KernelTiming t = g_timing;
    g_timing = KernelTiming{nullptr, nullptr};
    return t;
}

hipError_t launch_gemm_mfma_fp4_p1(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_fp4_p2(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_fp4_p3(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_mfma_fp4_p4(const GemmArgs &g, hipStream_t stream);

// The fp32 accumulator runs from the recovery terms to C through integer partial sums; all of them are
// below 4 K' (2^p - 1)(2^q - 1) in magnitude, which must stay below 2^24 for the sums to be exact.
bool gemm_mfma_fp4_supported(const GemmArgs &g)
{
    if (g.p < 1 || g.p > 4 || g.q < 1 || g.q > 4) return false;
    const int64_t unit = (int64_t)((1 << g.p) - 1) * ((1 << g.q) - 1);
    return 4 * g.nkb * kKBlock * unit < (1 << 24);
}

hipError_t launch_gemm_mfma_fp4(const GemmArgs &g, hipStream_t stream)
{
    switch (g.p) {
    case 1: return launch_gemm_mfma_fp4_p1(g, stream);
    case 2: return launch_gemm_mfma_fp4_p2(g, stream);
    case 3: return launch_gemm_mfma_fp4_p3(g, stream);
    case 4: return launch_gemm_mfma_fp4_p4(g, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace apmm
