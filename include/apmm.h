/*
 * apmm.h - C ABI of the bipolar-INT arbitrary-precision GEMM library for MI355X (gfx950).
 *
 * The library computes C = A * W^T where A (M x K activations, p bits) and W (N x K
 * weights, q bits) hold bipolar-INT codes: bit i of a code contributes (2*bit - 1) * 2^i
 * (paper Sec. 3.1, Eq. 1), so an n-bit code u has the value 2u - (2^n - 1).
 * The operands are first decomposed into 1-bit planes, reassembled into 32-bit words
 * and concatenated into one buffer (paper Sec. 4.1, steps 1-3: apmm_pack_*); the GEMM
 * multiplies the planes and recovers C = sum_i sum_j 2^(i+j) * D_ij on chip, never in
 * global memory (paper Sec. 3.2 and Sec. 4.2: apmm_gemm).
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates
 *    no device memory and keeps no state besides a thread-local error string.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is
 *    enqueued asynchronously on it; the call returns once the kernels are launched.
 *  - Argument errors are detected on the host before any launch and leave the outputs
 *    untouched.
 *  - Codes are one uint8 per element, row-major with K contiguous; only the low `bits`
 *    bits are significant, higher bits are ignored.
 *  - Packed buffers are opaque.  Their size is apmm_packed_bytes() for weights and
 *    apmm_packed_activation_bytes() for activations; the only contractual property is
 *    apmm_unpack*(apmm_pack_*(x)) == x on the low `bits` bits.  They must be
 *    16-byte aligned (any hipMalloc / PyTorch allocation is).
 */
#ifndef APMM_H
#define APMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    APMM_OK = 0,
    APMM_ERR_INVALID_ARG = 1, /* null pointer, negative size, bits outside [1, 8], misaligned buffer */
    APMM_ERR_UNSUPPORTED = 2, /* valid request that no kernel in this build covers */
    APMM_ERR_OVERFLOW = 3,    /* K * (2^p - 1) * (2^q - 1) does not fit the 32-bit output */
    APMM_ERR_WORKSPACE = 4,   /* workspace missing or smaller than the call needs (apmm_gemm_from_codes) */
    APMM_ERR_HIP = 5          /* a HIP call failed; text in apmm_last_error() */
} apmm_status;

/* Kernel selection for apmm_gemm_ex.  apmm_gemm uses APMM_ALGO_AUTO. */
typedef enum {
    APMM_ALGO_AUTO = 0,
    APMM_ALGO_VALU_POPCOUNT = 1, /* plane pairs by XOR + popcount on the vector ALU, D_ij = K - 2*popc */
    APMM_ALGO_DECODE = 3,        /* small-M weight-streaming kernels: on the matrix unit for p, q <= 4 and M <= 64 (unpacked
                                    activation codes of 3 and 4 bits: M <= 32); else XOR + popcount for M <= 16, q <= 4 and p not 3 or 4 */
    APMM_ALGO_MFMA_FP4 = 4,      /* plane groups recombined to E2M1 codes in registers, f8f6f4 MFMA, exact fp32 accumulate
                                    (p, q <= 4 and 4 * roundup(K,512) * (2^p-1)(2^q-1) < 2^24); the large-tile kernel, every
                                    wave sweeping all of K */
    APMM_ALGO_DECODE_VALU = 5,   /* the XOR + popcount small-M kernel whatever the widths (M <= 16, q <= 4, p not 3 or 4):
                                    design B at decode shapes, for comparison */
    /* Ablation for the claim of paper Sec. 4.2 (p <= 2, q <= 4, same K bound as APMM_ALGO_MFMA_FP4); planes as +-1
       operands on the matrix unit: */
    APMM_ALGO_PLANE_PAIRS_GLOBAL = 6, /* the scheme the paper argues against: one plane pair per workgroup, its 32-bit
                                    product D_ij to global memory, then a pass that shifts and adds them into C.
                                    Needs `workspace` of p * q * M * N * 4 bytes (16-byte aligned), else
                                    APMM_ERR_WORKSPACE */
    APMM_ALGO_PLANES_REGISTERS = 7, /* one tile per workgroup, an accumulator per plane pair, shift-and-add in registers
                                    (the paper's recovery-oriented scheme) */
    APMM_ALGO_MFMA_KSPLIT = 8    /* APMM_ALGO_MFMA_FP4 with the K partition of paper Sec. 4.2 taken across the four waves of
                                    a workgroup as well: every wave holds the whole workgroup tile for a quarter of K, the
                                    partial tiles are added in LDS (chosen by AUTO for outputs of one round of tiles and long K) */
} apmm_algo;

/* Bytes of the packed form of a rows x K operand of `bits`-bit codes (paper Sec. 4.1:
 * `bits` one-bit planes in 32-bit words, concatenated, plus one int32 per row).  Rows are padded
 * to a multiple of 32 and K to a multiple of 512.  Returns 0 for invalid arguments. */
size_t apmm_packed_bytes(int64_t rows, int64_t K, int bits);

/* Bytes of the packed form of M x K activations of p bits.  Equal to apmm_packed_bytes(M, K, p) except
 * for p = 3 and 4, whose codes are stored as 6-bit fields, the matrix unit's own operand form, so that
 * the GEMM needs neither a second sweep of K nor an expansion for them. */
size_t apmm_packed_activation_bytes(int64_t M, int64_t K, int p);

/* Bytes of scratch apmm_gemm needs for this problem (may be 0). */
size_t apmm_workspace_bytes(int64_t M, int64_t N, int64_t K, int p, int q);

/* Paper Sec. 4.1 (matrix decomposition and reassembly) for the weight matrix.
 *   w_codes  : device, N x K uint8 codes, row-major.
 *   w_packed : device, apmm_packed_bytes(N, K, q) bytes, written entirely.
 * N == 0 is allowed (nothing is done).  K must be >= 1. */
apmm_status apmm_pack_weights(const uint8_t *w_codes, int64_t N, int64_t K, int q,
                              void *w_packed, void *stream);

/* Same transform for the activation matrix (M x K codes of p bits); meant to run online,
 * directly before apmm_gemm on the same stream.  a_packed: apmm_packed_activation_bytes(M, K, p) bytes. */
apmm_status apmm_pack_activations(const uint8_t *a_codes, int64_t M, int64_t K, int p,
                                  void *a_packed, void *stream);

/* Paper Sec. 3.1 (the feature matrix is quantised onto the symmetric bipolar-INT grid) fused with the
 * packing of Sec. 4.1, for activations that arrive as binary16 numbers: one pass instead of writing and
 * re-reading one code byte per element.  Per row (token) m:
 *   a_scale[m] = max_k |x[m][k]| / (2^p - 1), correctly rounded to binary16 (nearest, ties to even)
 *   code       = (v + 2^p - 1) / 2, v = the odd integer of [-(2^p - 1), 2^p - 1] nearest to x / a_scale[m],
 *                the upper one on a tie
 * decided as in exact arithmetic on the binary16 values (an element exactly on a cell border
 * x = 2 c a_scale[m] always lands in the upper cell); a row whose scale rounds to zero gets the code of +1
 * everywhere.  The result is the packed operand apmm_pack_activations would give
 * for those codes, and a_scale is the per-token scale for apmm_gemm's fp16 epilogue.
 *   x_f16    : device, M x K binary16 bit patterns, row-major, finite values
 *   a_packed : device, apmm_packed_activation_bytes(M, K, p) bytes, written entirely
 *   a_scale  : device, M binary16 bit patterns, written */
apmm_status apmm_quantize_pack_activations(const uint16_t *x_f16, int64_t M, int64_t K, int p,
                                           void *a_packed, uint16_t *a_scale, void *stream);

/* Inverse of apmm_pack_weights (test aid): writes rows x K uint8 codes. */
apmm_status apmm_unpack(const void *packed, int64_t rows, int64_t K, int bits,
                        uint8_t *codes, void *stream);
/* Inverse of apmm_pack_activations (test aid): writes M x K uint8 codes. */
apmm_status apmm_unpack_activations(const void *a_packed, int64_t M, int64_t K, int p,
                                    uint8_t *codes, void *stream);

/* Paper Sec. 3.2 (bit-wise MatMul reconstitution) with the recovery of Sec. 4.2 kept on chip.
 *   a_packed : device, packed M x K activations of p bits (from apmm_pack_activations)
 *   w_packed : device, packed N x K weights of q bits     (from apmm_pack_weights)
 *   c_i32    : device, M x N row-major int32 result, or NULL
 *   c_f16    : device, M x N row-major IEEE binary16 bit patterns of
 *              C[m][n] * a_scale[m] * w_scale[n] (product in fp32, one rounding to
 *              nearest-even at the end; a product beyond the binary16 range, |x| >= 65520,
 *              becomes an infinity of its sign, as IEEE 754 rounding has it), or NULL
 *   w_scale  : device, N binary16 per-output-channel scales, or NULL (= 1)
 *   a_scale  : device, M binary16 per-token scales, or NULL (= 1)
 *   workspace: device scratch of at least apmm_workspace_bytes() bytes (may be NULL if 0; only
 *              APMM_ALGO_PLANE_PAIRS_GLOBAL of apmm_gemm_ex uses one)
 * At least one of c_i32 / c_f16 must be non-NULL.  M == 0 or N == 0 returns APMM_OK
 * without a launch.  Returns APMM_ERR_OVERFLOW if roundup(K,512)*(2^p-1)*(2^q-1) > INT32_MAX. */
apmm_status apmm_gemm(int64_t M, int64_t N, int64_t K, int p, int q,
                      const void *a_packed, const void *w_packed,
                      int32_t *c_i32, uint16_t *c_f16,
                      const uint16_t *w_scale, const uint16_t *a_scale,
                      void *workspace, size_t workspace_bytes, void *stream);

/* apmm_gemm with an explicit kernel choice (used to compare the two designs).
 * Returns APMM_ERR_UNSUPPORTED if `algo` does not cover the request. */
apmm_status apmm_gemm_ex(int64_t M, int64_t N, int64_t K, int p, int q,
                         const void *a_packed, const void *w_packed,
                         int32_t *c_i32, uint16_t *c_f16,
                         const uint16_t *w_scale, const uint16_t *a_scale,
                         void *workspace, size_t workspace_bytes, void *stream,
                         int algo);

/* apmm_gemm taking the activation codes as they are: the preprocessing of paper Sec. 4.1 (decomposition,
 * reassembly, concatenation) for the activations and the bit-wise MatMul of Sec. 3.2 in one call, as an
 * inference engine meets them (Sec. 5.2: the activations of a layer are produced online).  `a_codes` is
 * the device M x K row-major uint8 matrix that apmm_pack_activations would take (bits above p are
 * ignored, no alignment needed).  Result and all other arguments as in apmm_gemm.
 *   - For a few tokens the small-M kernels regroup the codes into the packed form on their way into
 *     on-chip memory: one launch, no packed buffer.  The separate packing launch costs as much as such a
 *     GEMM.  Taken when the small-M kernels cover the shape (M <= 16 with q <= 4 and p not 3 or 4, or
 *     M <= 64 with p, q <= 2) and M <= 16 or M * N <= 65536.
 *   - Otherwise the codes are packed into `workspace` (device, 16-byte aligned, at least
 *     apmm_packed_activation_bytes(M, K, p) bytes, overwritten) and apmm_gemm runs on that: two launches.
 * Without such a workspace the call still takes the one-launch path wherever the small-M kernels cover the
 * shape, and returns APMM_ERR_WORKSPACE (nothing launched) where they do not. */
apmm_status apmm_gemm_from_codes(int64_t M, int64_t N, int64_t K, int p, int q,
                                 const uint8_t *a_codes, const void *w_packed,
                                 int32_t *c_i32, uint16_t *c_f16,
                                 const uint16_t *w_scale, const uint16_t *a_scale,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): apmm_gemm_from_codes without the workspace argument.  The packed activations go into
 * a buffer of APMM_NOALLOC_MAX_PACKED_BYTES bytes that is part of the library's device code (one per GPU, held
 * until the process ends); the call allocates and frees nothing.  Arguments, result and kernel choice as in
 * apmm_gemm_from_codes with a workspace of that size.
 *   - Returns APMM_ERR_WORKSPACE (nothing launched) when apmm_packed_activation_bytes(M, K, p) exceeds
 *     APMM_NOALLOC_MAX_PACKED_BYTES, whether or not the shape would have needed the buffer.
 *   - Every call on one GPU uses that GPU's one buffer, from the packing launch to the end of the GEMM that
 *     follows it on `stream`: calls that overlap on one GPU (different streams, or different threads) race.
 *     Calls on one stream are ordered and safe.  Nothing in the buffer has to be cleared between calls: the
 *     packing writes every byte the GEMM reads. */
#define APMM_NOALLOC_MAX_PACKED_BYTES ((size_t)8 << 20)
apmm_status apmm_gemm_from_codes_noalloc(int64_t M, int64_t N, int64_t K, int p, int q,
                                         const uint8_t *a_codes, const void *w_packed,
                                         int32_t *c_i32, uint16_t *c_f16,
                                         const uint16_t *w_scale, const uint16_t *a_scale, void *stream);

/* One linear of a grouped call: C = A * W^T with the arguments of apmm_gemm. */
typedef struct apmm_problem {
    int64_t M, N, K;
    const void *a_packed;     /* device, packed M x K activations of p bits; ignored when a_codes is given */
    const void *w_packed;     /* device, packed N x K weights of q bits */
    int32_t *c_i32;           /* device, M x N, or NULL */
    uint16_t *c_f16;          /* device, M x N binary16 bit patterns, or NULL */
    const uint16_t *w_scale;  /* device, N, or NULL */
    const uint16_t *a_scale;  /* device, M, or NULL */
    const uint8_t *a_codes;   /* device, M x K unpacked activation codes as for apmm_gemm_from_codes, or NULL */
} apmm_problem;

/* Paper Sec. 5.2 setting (the linears of a decoder layer, each the MatMul of Sec. 3.2): several independent
 * GEMMs of equal p and q with as few launches as possible (for callers whose
 * linears are small enough that the launch, not the data, bounds them: the q/k/v or gate/up
 * projections of one decoder layer at a few tokens share their activations and can go in one launch).
 * `problems` is a HOST array of `count` entries, read before the call returns.  Each entry obeys the
 * rules of apmm_gemm and gives the same result as apmm_gemm on it.  Small-M problems that the same
 * small-M kernel covers are launched eight at a time; all others are launched one by one.  The outputs
 * of different entries must not overlap.  At most 256 entries.  On an argument error nothing is launched.
 * An entry with a_codes takes its activations unpacked, as apmm_gemm_from_codes does in its one-launch
 * form (no packing launch, no packed buffer); such an entry must be a shape the small-M kernels cover,
 * else the call returns APMM_ERR_UNSUPPORTED.  Entries with and without a_codes do not share a launch. */
apmm_status apmm_gemm_grouped(int count, const apmm_problem *problems, int p, int q,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Measurement aid.  The next apmm_gemm / apmm_gemm_ex / apmm_gemm_from_codes call of the calling thread, if it
 * runs the large-tile MFMA kernel or a small-M kernel in one launch, attaches the two hipEvent_t (created by the
 * caller; either may be NULL) to that kernel's dispatch itself (hipExtLaunchKernel): afterwards they hold the
 * kernel's own begin and end, without the dispatch gaps that events recorded before and after the call include.
 * A call that runs the general XOR/popcount kernel drops them. */
apmm_status apmm_time_next_gemm(void *start_event, void *stop_event);

/* Measurement aid.  Name, with its template arguments, of the GEMM kernel that the last GEMM call of the calling
 * thread launched ("" before the first), e.g. "gemm_mfma_direct_kernel<2,1,4,4,3>" (activation bits, weight bits,
 * wave tile in 32-row and 32-column blocks, store phases).  The string is overwritten by the next GEMM call. */
const char *apmm_last_gemm_kernel(void);

const char *apmm_status_string(apmm_status status);
/* Text of the last error on the calling thread ("" if none). */
const char *apmm_last_error(void);
int apmm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* APMM_H */
