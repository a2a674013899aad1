// C ABI of the library (include/apmm.h): argument checks and kernel dispatch.  No kernel
// lives here and nothing is allocated.
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/apmm.h"
#include "apmm_kernels.h"

namespace {

thread_local char g_error[256] = "";

apmm_status fail(apmm_status st, const char *msg)
{
    std::snprintf(g_error, sizeof(g_error), "%s", msg);
    return st;
}

apmm_status fail_hip(hipError_t e, const char *where)
{
    std::snprintf(g_error, sizeof(g_error), "%s: %s", where, hipGetErrorString(e));
    return APMM_ERR_HIP;
}

bool bits_ok(int bits) { return bits >= 1 && bits <= 8; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

apmm_status pack_common(const uint8_t *codes, int64_t rows, int64_t K, int bits, bool field, void *packed,
                        void *stream, const char *what)
{
    if (rows < 0 || K < 1 || !bits_ok(bits)) return fail(APMM_ERR_INVALID_ARG, "pack: rows < 0, K < 1 or bits outside [1, 8]");
    if (rows == 0) return APMM_OK;
    if (!codes || !packed) return fail(APMM_ERR_INVALID_ARG, "pack: null pointer");
    if (!aligned16(packed)) return fail(APMM_ERR_INVALID_ARG, "pack: packed buffer must be 16-byte aligned");
    hipError_t e = apmm::launch_pack(codes, rows, K, bits, field, static_cast<uint32_t *>(packed),
                                     static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, what);
    return APMM_OK;
}

}  // namespace

extern "C" {

size_t apmm_packed_bytes(int64_t rows, int64_t K, int bits)
{
    if (rows < 0 || K < 1 || !bits_ok(bits)) return 0;
    const int64_t rows_p = apmm::round_up(rows, apmm::kRowBlock);
    const int64_t k_p = apmm::round_up(K, apmm::kKPad);
    return (size_t)rows_p * (size_t)k_p / 8u * (size_t)bits + (size_t)rows_p * 4u;  // planes + row sums
}

size_t apmm_packed_activation_bytes(int64_t M, int64_t K, int p)
{
    if (M < 0 || K < 1 || !bits_ok(p)) return 0;
    const int64_t rows_p = apmm::round_up(M, apmm::kRowBlock);
    const int64_t k_p = apmm::round_up(K, apmm::kKPad);
    return (size_t)rows_p * (size_t)k_p / 8u * (size_t)apmm::activation_slots(p) + (size_t)rows_p * 4u;
}

size_t apmm_workspace_bytes(int64_t, int64_t, int64_t, int, int) { return 0; }

apmm_status apmm_pack_weights(const uint8_t *w_codes, int64_t N, int64_t K, int q, void *w_packed, void *stream)
{
    return pack_common(w_codes, N, K, q, false, w_packed, stream, "apmm_pack_weights");
}

apmm_status apmm_pack_activations(const uint8_t *a_codes, int64_t M, int64_t K, int p, void *a_packed,
                                  void *stream)
{
    return pack_common(a_codes, M, K, p, apmm::activation_field_form(p), a_packed, stream, "apmm_pack_activations");
}

apmm_status apmm_quantize_pack_activations(const uint16_t *x_f16, int64_t M, int64_t K, int p, void *a_packed,
                                           uint16_t *a_scale, void *stream)
{
    if (M < 0 || K < 1 || !bits_ok(p)) return fail(APMM_ERR_INVALID_ARG, "quantize_pack: M < 0, K < 1 or bits outside [1, 8]");
    if (M == 0) return APMM_OK;
    if (!x_f16 || !a_packed || !a_scale) return fail(APMM_ERR_INVALID_ARG, "quantize_pack: null pointer");
    if (!aligned16(a_packed)) return fail(APMM_ERR_INVALID_ARG, "quantize_pack: packed buffer must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(x_f16) & 1u) || (reinterpret_cast<uintptr_t>(a_scale) & 1u))
        return fail(APMM_ERR_INVALID_ARG, "quantize_pack: misaligned binary16 buffer");
    hipError_t e = apmm::launch_quantize_pack(x_f16, M, K, p, apmm::activation_field_form(p),
                                              static_cast<uint32_t *>(a_packed), a_scale,
                                              static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "apmm_quantize_pack_activations");
    return APMM_OK;
}

namespace {
apmm_status unpack_common(const void *packed, int64_t rows, int64_t K, int bits, bool field, uint8_t *codes, void *stream)
{
    if (rows < 0 || K < 1 || !bits_ok(bits)) return fail(APMM_ERR_INVALID_ARG, "unpack: rows < 0, K < 1 or bits outside [1, 8]");
    if (rows == 0) return APMM_OK;
    if (!codes || !packed) return fail(APMM_ERR_INVALID_ARG, "unpack: null pointer");
    if (!aligned16(packed)) return fail(APMM_ERR_INVALID_ARG, "unpack: packed buffer must be 16-byte aligned");
    hipError_t e = apmm::launch_unpack(static_cast<const uint32_t *>(packed), rows, K, bits, field, codes,
                                       static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "apmm_unpack");
    return APMM_OK;
}
}  // namespace

apmm_status apmm_unpack(const void *packed, int64_t rows, int64_t K, int bits, uint8_t *codes, void *stream)
{
    return unpack_common(packed, rows, K, bits, false, codes, stream);
}

apmm_status apmm_unpack_activations(const void *a_packed, int64_t M, int64_t K, int p, uint8_t *codes, void *stream)
{
    return unpack_common(a_packed, M, K, p, apmm::activation_field_form(p), codes, stream);
}

}  // extern "C"

namespace {

// Argument checks of one GEMM; fills `g`.  `empty` is set when M == 0 or N == 0 (nothing to launch).
apmm_status check_gemm(int64_t M, int64_t N, int64_t K, int p, int q, const void *a_packed, const void *w_packed,
                       int32_t *c_i32, uint16_t *c_f16, const uint16_t *w_scale, const uint16_t *a_scale,
                       apmm::GemmArgs &g, bool &empty, bool a_is_codes = false)
{
    empty = false;
    if (M < 0 || N < 0 || K < 1 || !bits_ok(p) || !bits_ok(q))
        return fail(APMM_ERR_INVALID_ARG, "gemm: M < 0, N < 0, K < 1 or bits outside [1, 8]");
    const int64_t k_p = apmm::round_up(K, apmm::kKPad);
    const int64_t unit = (int64_t)((1 << p) - 1) * (int64_t)((1 << q) - 1);
    if (k_p > INT32_MAX / unit) return fail(APMM_ERR_OVERFLOW, "gemm: K * (2^p - 1) * (2^q - 1) exceeds the 32-bit output");
    if (M == 0 || N == 0) {
        empty = true;
        return APMM_OK;
    }
    if (!a_packed || !w_packed) return fail(APMM_ERR_INVALID_ARG, "gemm: null operand");
    if (!c_i32 && !c_f16) return fail(APMM_ERR_INVALID_ARG, "gemm: no output requested");
    if ((!a_is_codes && !aligned16(a_packed)) || !aligned16(w_packed))
        return fail(APMM_ERR_INVALID_ARG, "gemm: packed operands must be 16-byte aligned");
    if ((c_i32 && (reinterpret_cast<uintptr_t>(c_i32) & 3u)) || (c_f16 && (reinterpret_cast<uintptr_t>(c_f16) & 1u)))
        return fail(APMM_ERR_INVALID_ARG, "gemm: misaligned output");
    g.M = M; g.N = N; g.K = K;
    g.nkb = k_p / apmm::kKBlock;
    g.p = p; g.q = q;
    g.w = static_cast<const uint32_t *>(w_packed);
    if (a_is_codes) {  // the small-M kernels pack the codes themselves and take the row sums on the way
        g.a = nullptr;
        g.a_sum = nullptr;
        g.a_codes = static_cast<const uint8_t *>(a_packed);
    } else {
        g.a = static_cast<const uint32_t *>(a_packed);
        g.a_sum = reinterpret_cast<const int32_t *>(
            g.a + apmm::row_sum_word(apmm::round_up(M, apmm::kRowBlock), g.nkb, apmm::activation_slots(p)));
        g.a_codes = nullptr;
    }
    g.w_sum = reinterpret_cast<const int32_t *>(g.w + apmm::row_sum_word(apmm::round_up(N, apmm::kRowBlock), g.nkb, q));
    g.c_i32 = c_i32; g.c_f16 = c_f16;
    g.w_scale = w_scale; g.a_scale = a_scale;
    return APMM_OK;
}

constexpr int kMaxProblems = 256;  // entries of one apmm_gemm_grouped call

apmm_status run_gemm(const apmm::GemmArgs &g, int algo, hipStream_t s, void *workspace = nullptr, size_t workspace_bytes = 0)
{
    if (algo == APMM_ALGO_AUTO) {
        // (33 - 64 tokens at more than 8192 channels: the small-M kernel needs a second round of its one-per-CU workgroups
        // there, 10.0 us at 11008 x 4096, and the K-split kernel's 86 tiles take 7.9 - 8.6 us)
        if (apmm::gemm_decode_supported(g) && !(g.M > 32 && g.N > 8192 && !g.a_codes && apmm::gemm_mfma_ksplit_pays(g)))
            algo = APMM_ALGO_DECODE;
        else if (apmm::gemm_mfma_fp4_supported(g)) algo = apmm::gemm_mfma_ksplit_pays(g) ? APMM_ALGO_MFMA_KSPLIT : APMM_ALGO_MFMA_FP4;
        else algo = APMM_ALGO_VALU_POPCOUNT;
    }
    if (algo == APMM_ALGO_VALU_POPCOUNT || algo == APMM_ALGO_PLANE_PAIRS_GLOBAL || algo == APMM_ALGO_PLANES_REGISTERS)
        (void)apmm::take_kernel_timing();  // those kernels take no timing events
    hipError_t e;
    switch (algo) {
    case APMM_ALGO_VALU_POPCOUNT:
        e = apmm::launch_gemm_valu(g, s);
        break;
    case APMM_ALGO_MFMA_FP4:
        if (!apmm::gemm_mfma_fp4_supported(g)) return fail(APMM_ERR_UNSUPPORTED, "gemm: FP4 MFMA kernel covers p, q in 1..4 while 4 K (2^p - 1)(2^q - 1) < 2^24");
        e = apmm::launch_gemm_mfma_fp4(g, s);
        break;
    case APMM_ALGO_MFMA_KSPLIT:
        if (!apmm::gemm_mfma_ksplit_supported(g)) return fail(APMM_ERR_UNSUPPORTED, "gemm: the K-split MFMA kernel covers p, q in 1..4 while 4 K (2^p - 1)(2^q - 1) < 2^24");
        e = apmm::launch_gemm_mfma_ksplit(g, s);
        break;
    case APMM_ALGO_DECODE:
        if (!apmm::gemm_decode_supported(g)) return fail(APMM_ERR_UNSUPPORTED, "gemm: decode kernel does not cover this request");
        e = apmm::launch_gemm_decode(g, s);
        break;
    case APMM_ALGO_PLANE_PAIRS_GLOBAL:
    case APMM_ALGO_PLANES_REGISTERS: {
        if (!apmm::gemm_ablation_supported(g))
            return fail(APMM_ERR_UNSUPPORTED, "gemm: the plane kernels cover p <= 2, q <= 4 while 4 K (2^p - 1)(2^q - 1) < 2^24");
        int32_t *pairs = nullptr;
        if (algo == APMM_ALGO_PLANE_PAIRS_GLOBAL) {
            if (!workspace || workspace_bytes < apmm::gemm_ablation_pairs_bytes(g))
                return fail(APMM_ERR_WORKSPACE, "gemm: the plane-pair scheme needs a workspace of p * q * M * N * 4 bytes");
            if (!aligned16(workspace)) return fail(APMM_ERR_INVALID_ARG, "gemm: workspace must be 16-byte aligned");
            pairs = static_cast<int32_t *>(workspace);
        }
        e = apmm::launch_gemm_ablation(g, pairs, s);
        break;
    }
    case APMM_ALGO_DECODE_VALU:
        if (!apmm::gemm_decode_valu_supported(g)) return fail(APMM_ERR_UNSUPPORTED, "gemm: the XOR/popcount small-M kernel does not cover this request");
        e = apmm::launch_gemm_decode_valu(g, s);
        break;
    default:
        return fail(APMM_ERR_INVALID_ARG, "gemm: unknown algo");
    }
    if (e != hipSuccess) return fail_hip(e, "apmm_gemm");
    return APMM_OK;
}

}  // namespace

extern "C" {

apmm_status apmm_gemm_ex(int64_t M, int64_t N, int64_t K, int p, int q, const void *a_packed,
                         const void *w_packed, int32_t *c_i32, uint16_t *c_f16, const uint16_t *w_scale,
                         const uint16_t *a_scale, void *workspace, size_t workspace_bytes, void *stream,
                         int algo)
{
    if (algo != APMM_ALGO_AUTO && algo != APMM_ALGO_VALU_POPCOUNT && algo != APMM_ALGO_DECODE && algo != APMM_ALGO_MFMA_FP4 &&
        algo != APMM_ALGO_DECODE_VALU && algo != APMM_ALGO_PLANE_PAIRS_GLOBAL && algo != APMM_ALGO_PLANES_REGISTERS &&
        algo != APMM_ALGO_MFMA_KSPLIT)
        return fail(APMM_ERR_INVALID_ARG, "gemm: unknown algo");
    apmm::GemmArgs g;
    bool empty;
    const apmm_status st = check_gemm(M, N, K, p, q, a_packed, w_packed, c_i32, c_f16, w_scale, a_scale, g, empty);
    if (st != APMM_OK || empty) return st;
    return run_gemm(g, algo, static_cast<hipStream_t>(stream), workspace, workspace_bytes);
}

apmm_status apmm_gemm_from_codes(int64_t M, int64_t N, int64_t K, int p, int q, const uint8_t *a_codes,
                                 const void *w_packed, int32_t *c_i32, uint16_t *c_f16, const uint16_t *w_scale,
                                 const uint16_t *a_scale, void *workspace, size_t workspace_bytes, void *stream)
{
    apmm::GemmArgs g;
    bool empty;
    const apmm_status st =
        check_gemm(M, N, K, p, q, a_codes, w_packed, c_i32, c_f16, w_scale, a_scale, g, empty, /*a_is_codes=*/true);
    if (st != APMM_OK || empty) return st;
    if (workspace && !aligned16(workspace)) return fail(APMM_ERR_INVALID_ARG, "gemm_from_codes: workspace must be 16-byte aligned");
    const bool fused_ok = apmm::gemm_decode_supported(g);
    const bool room = workspace && workspace_bytes >= apmm_packed_activation_bytes(M, K, p);
    // Every workgroup of the small-M kernels loads all M x K codes for itself: that beats a packing launch
    // (2.5 - 3 us) up to 16 tokens at every width measured (16 tokens x 11008 channels: 7.3 us in one launch, 7.2 us
    // in two), and for more tokens while M x N is small.
    // (3- and 4-bit activations: turning codes into 6-bit fields costs more, the one-launch form wins up to 8 tokens:
    // W2A4 at 11008 x 4096 6.0 / 7.5 / 9.6 us for 1 / 8 / 16 tokens against about 8 - 8.8 us in two launches)
    const bool fused_pays = apmm::activation_field_form(p) ? (M <= 8 || M * N <= 65536) : (M <= 16 || M * N <= 65536);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fused_ok && (fused_pays || !room)) {
        const hipError_t e = apmm::launch_gemm_decode(g, s);
        if (e != hipSuccess) return fail_hip(e, "apmm_gemm_from_codes");
        return APMM_OK;
    }
    if (!room)
        return fail(APMM_ERR_WORKSPACE, "gemm_from_codes: this shape needs a workspace of apmm_packed_activation_bytes(M, K, p) bytes");
    const apmm_status ps = pack_common(a_codes, M, K, p, apmm::activation_field_form(p), workspace, stream, "apmm_gemm_from_codes");
    if (ps != APMM_OK) return ps;
    const apmm_status cs = check_gemm(M, N, K, p, q, workspace, w_packed, c_i32, c_f16, w_scale, a_scale, g, empty);
    if (cs != APMM_OK) return cs;
    return run_gemm(g, APMM_ALGO_AUTO, s);
}

}  // extern "C"

namespace {

// Packed activations of apmm_gemm_from_codes_noalloc: one array per GPU, held until the process ends.  In host
// code the array's name is only a stand-in: the device address is looked up once per device (below) and that
// pointer is what kernels and every other call get.
constexpr size_t kScratchBytes = APMM_NOALLOC_MAX_PACKED_BYTES;
__device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};  // by device ordinal; written once under the mutex

apmm_status scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "apmm_gemm_from_codes_noalloc: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(APMM_ERR_UNSUPPORTED, "gemm_from_codes_noalloc: device ordinal beyond 63");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // this device's copy of the array
        if (e != hipSuccess) return fail_hip(e, "apmm_gemm_from_codes_noalloc: hipGetSymbolAddress");
        if (!ptr) return fail(APMM_ERR_HIP, "gemm_from_codes_noalloc: no device address for the scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return APMM_OK;
}

}  // namespace

extern "C" {

apmm_status apmm_gemm_from_codes_noalloc(int64_t M, int64_t N, int64_t K, int p, int q, const uint8_t *a_codes,
                                         const void *w_packed, int32_t *c_i32, uint16_t *c_f16,
                                         const uint16_t *w_scale, const uint16_t *a_scale, void *stream)
{
    if (M < 0 || K < 1 || !bits_ok(p))
        return fail(APMM_ERR_INVALID_ARG, "gemm: M < 0, N < 0, K < 1 or bits outside [1, 8]");
    const size_t need = apmm_packed_activation_bytes(M, K, p);
    if (need > kScratchBytes) {
        std::snprintf(g_error, sizeof(g_error),
                      "gemm_from_codes_noalloc: the packed activations of this call take %zu bytes, the built-in "
                      "buffer holds %zu (use apmm_gemm_from_codes with a workspace)", need, kScratchBytes);
        return APMM_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    const apmm_status st = scratch_of_current_device(&ws);
    if (st != APMM_OK) return st;
    return apmm_gemm_from_codes(M, N, K, p, q, a_codes, w_packed, c_i32, c_f16, w_scale, a_scale, ws, kScratchBytes,
                                stream);
}

apmm_status apmm_time_next_gemm(void *start_event, void *stop_event)
{
    apmm::set_kernel_timing(static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event));
    return APMM_OK;
}

apmm_status apmm_gemm_grouped(int count, const apmm_problem *problems, int p, int q, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (count < 0 || (count > 0 && !problems)) return fail(APMM_ERR_INVALID_ARG, "gemm_grouped: bad problem list");
    if (count > kMaxProblems) return fail(APMM_ERR_INVALID_ARG, "gemm_grouped: more than 256 problems");
    // every entry is checked before anything is launched
    static thread_local apmm::GemmArgs args[kMaxProblems];
    int live = 0;
    for (int i = 0; i < count; ++i) {
        const apmm_problem &pr = problems[i];
        bool empty;
        const bool codes = pr.a_codes != nullptr;
        const apmm_status st = check_gemm(pr.M, pr.N, pr.K, p, q, codes ? static_cast<const void *>(pr.a_codes) : pr.a_packed,
                                          pr.w_packed, pr.c_i32, pr.c_f16, pr.w_scale, pr.a_scale, args[live], empty, codes);
        if (st != APMM_OK) return st;
        if (codes && !empty && !apmm::gemm_decode_supported(args[live]))
            return fail(APMM_ERR_UNSUPPORTED, "gemm_grouped: an entry with a_codes must be a shape the small-M kernels cover");
        if (!empty) ++live;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int i = 0;
    while (i < live) {
        // longest run (up to kMaxGroup) that one small-M launch covers
        int run = 1;
        while (i + run < live && run < apmm::kMaxGroup && apmm::gemm_decode_group_supported(args + i, run + 1)) ++run;
        if (run > 1 || apmm::gemm_decode_group_supported(args + i, 1)) {
            hipError_t e = apmm::launch_gemm_decode_group(args + i, run, s);
            if (e != hipSuccess) return fail_hip(e, "apmm_gemm_grouped");
        } else {
            const apmm_status st = run_gemm(args[i], APMM_ALGO_AUTO, s);
            if (st != APMM_OK) return st;
        }
        i += run;
    }
    return APMM_OK;
}

apmm_status apmm_gemm(int64_t M, int64_t N, int64_t K, int p, int q, const void *a_packed, const void *w_packed,
                      int32_t *c_i32, uint16_t *c_f16, const uint16_t *w_scale, const uint16_t *a_scale,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    return apmm_gemm_ex(M, N, K, p, q, a_packed, w_packed, c_i32, c_f16, w_scale, a_scale, workspace,
                        workspace_bytes, stream, APMM_ALGO_AUTO);
}

const char *apmm_status_string(apmm_status status)
{
    switch (status) {
    case APMM_OK: return "ok";
    case APMM_ERR_INVALID_ARG: return "invalid argument";
    case APMM_ERR_UNSUPPORTED: return "unsupported";
    case APMM_ERR_OVERFLOW: return "result exceeds 32 bits";
    case APMM_ERR_WORKSPACE: return "workspace too small";
    case APMM_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

const char *apmm_last_error(void) { return g_error; }

const char *apmm_last_gemm_kernel(void) { return apmm::last_kernel(); }

int apmm_version(void) { return 100; }

}  // extern "C"
