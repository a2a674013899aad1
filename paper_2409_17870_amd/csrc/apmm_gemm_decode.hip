// Small-M (decode) kernel: placeholder until the weight-streaming kernel lands.
#include "apmm_kernels.h"

namespace apmm {
bool gemm_decode_supported(const GemmArgs &) { return false; }
hipError_t launch_gemm_decode(const GemmArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace apmm
