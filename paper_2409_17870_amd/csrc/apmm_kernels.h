// Host-side launchers of the library's kernels (internal; the public ABI is include/apmm.h).
#pragma once
#include <hip/hip_runtime.h>
#include "apmm_layout.h"

namespace apmm {

// Paper Sec. 4.1: decomposition into planes, reassembly into 32-bit words, concatenation.
// `field`: the field form of 3- and 4-bit activations instead of the group form (apmm_layout.h).
hipError_t launch_pack(const uint8_t *codes, int64_t rows, int64_t K, int bits, bool field, uint32_t *packed,
                       hipStream_t stream);
// Paper Sec. 3.1 + 4.1: per-row symmetric quantisation of binary16 features fused with the packing.
hipError_t launch_quantize_pack(const uint16_t *x, int64_t rows, int64_t K, int bits, bool field, uint32_t *packed,
                                uint16_t *scale, hipStream_t stream);
hipError_t launch_unpack(const uint32_t *packed, int64_t rows, int64_t K, int bits, bool field, uint8_t *codes,
                         hipStream_t stream);

// Design B: plane pairs by XOR + popcount on the vector ALU (any p, q in 1..8).
hipError_t launch_gemm_valu(const GemmArgs &args, hipStream_t stream);

// Design A: plane groups recombined into E2M1 / E2M3 codes in registers, f8f6f4 MFMA, exact fp32 accumulate
// (p, q in 1..4 while 4 K (2^p - 1)(2^q - 1) < 2^24).
bool gemm_mfma_fp4_supported(const GemmArgs &args);
hipError_t launch_gemm_mfma_fp4(const GemmArgs &args, hipStream_t stream);

// Design A with K split across the four waves of a workgroup (apmm_gemm_mfma_ksplit.h): for outputs of few
// tiles; same widths and exactness bound as above.
bool gemm_mfma_ksplit_supported(const GemmArgs &args);
bool gemm_mfma_ksplit_pays(const GemmArgs &args);  // the launch rule of launch_gemm_mfma_fp4 takes it for these
hipError_t launch_gemm_mfma_ksplit(const GemmArgs &args, hipStream_t stream);

// Ablation kernels for the claim of paper Sec. 4.2 (apmm_gemm_ablation.hip): the planes as +-1 operands on the
// matrix unit.  pairs != nullptr: every plane pair's product to global memory (p q M N int32 at `pairs`), then a
// recovery pass; pairs == nullptr: one tile per workgroup, recovery in registers.
bool gemm_ablation_supported(const GemmArgs &args);
size_t gemm_ablation_pairs_bytes(const GemmArgs &args);
hipError_t launch_gemm_ablation(const GemmArgs &args, int32_t *pairs, hipStream_t stream);

// Measurement aid: a pair of events that the next GEMM launch of the calling thread (large-tile MFMA kernel or
// small-M kernels) attaches to its kernel dispatch (hipExtLaunchKernel), so that they hold the kernel's own
// begin and end.
struct KernelTiming {
    hipEvent_t start, stop;
};
void set_kernel_timing(hipEvent_t start, hipEvent_t stop);
KernelTiming take_kernel_timing();  // returns the pair and clears it
// Measurement aid: name (with template arguments) of the GEMM kernel the calling thread launched last.
void note_kernel(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
const char *last_kernel();

// Small-M weight-streaming kernels: on the matrix unit for p, q <= 4 (M <= 64; unpacked activation codes of 3 and 4 bits: M <= 32), XOR/popcount for wider codes (M <= 16, p not 3 or 4).
bool gemm_decode_supported(const GemmArgs &args);
hipError_t launch_gemm_decode(const GemmArgs &args, hipStream_t stream);
// The XOR/popcount small-M kernel whatever the code widths (M <= 16, q <= 4): design B at decode shapes.
bool gemm_decode_valu_supported(const GemmArgs &args);
hipError_t launch_gemm_decode_valu(const GemmArgs &args, hipStream_t stream);
// Up to kMaxGroup small-M problems of equal p, q in one launch; they must all be covered by the same
// kernel variant (gemm_decode_group_supported).
bool gemm_decode_group_supported(const GemmArgs *args, int count);
hipError_t launch_gemm_decode_group(const GemmArgs *args, int count, hipStream_t stream, bool xor_only = false);

}  // namespace apmm
