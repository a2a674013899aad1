"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, sizes are right and argument errors are reported before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "apmm.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2409_17870_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(apmm_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2409_17870_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_single_hip_runtime_in_process(lib):
    """The library must bind to the HIP runtime PyTorch already loaded, not bring a second one."""
    paths = set()
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                paths.add(line.split()[-1])
    assert len(paths) == 1, paths


def test_packed_bytes(lib):
    assert lib.apmm_packed_bytes(32, 512, 1) == 32 * 512 // 8 + 32 * 4  # planes + one int32 code sum per row
    assert lib.apmm_packed_bytes(1, 1, 1) == 32 * 512 // 8 + 32 * 4  # padded to 32 rows x 512 k
    assert lib.apmm_packed_bytes(4096, 4096, 2) == 4096 * 4096 * 2 // 8 + 4096 * 4
    assert lib.apmm_packed_bytes(33, 129, 3) == 64 * 512 * 3 // 8 + 64 * 4
    # activations of 3 and 4 bits are stored as 6-bit fields, all others like weights
    assert lib.apmm_packed_activation_bytes(33, 129, 3) == 64 * 512 * 6 // 8 + 64 * 4
    assert lib.apmm_packed_activation_bytes(33, 129, 4) == 64 * 512 * 6 // 8 + 64 * 4
    for bits in (1, 2, 5, 8):
        assert lib.apmm_packed_activation_bytes(33, 129, bits) == lib.apmm_packed_bytes(33, 129, bits)
    assert lib.apmm_packed_bytes(0, 128, 2) == 0
    assert lib.apmm_packed_bytes(8, 128, 0) == 0 and lib.apmm_packed_bytes(8, 128, 9) == 0
    assert lib.apmm_packed_bytes(-1, 128, 2) == 0 and lib.apmm_packed_bytes(8, 0, 2) == 0
    assert lib.apmm_version() >= 100


def _gemm(lib, M, N, K, p, q, a=0x1000, w=0x2000, c=0x3000, f=None, algo=0):
    return lib.apmm_gemm_ex(M, N, K, p, q, a, w, c, f, None, None, None, 0, None, algo)


def test_argument_errors_come_before_any_launch(lib):
    INVALID, UNSUPPORTED, OVERFLOW = 1, 2, 3
    assert _gemm(lib, 4, 4, 128, 0, 1) == INVALID
    assert _gemm(lib, 4, 4, 128, 1, 9) == INVALID
    assert _gemm(lib, -1, 4, 128, 1, 1) == INVALID
    assert _gemm(lib, 4, 4, 0, 1, 1) == INVALID
    assert _gemm(lib, 4, 4, 128, 1, 1, a=None) == INVALID
    assert _gemm(lib, 4, 4, 128, 1, 1, c=None) == INVALID          # no output requested
    assert _gemm(lib, 4, 4, 128, 1, 1, a=0x1004) == INVALID         # misaligned packed operand
    assert _gemm(lib, 4, 4, 128, 1, 1, algo=9) == INVALID
    assert _gemm(lib, 64, 64, 128, 5, 1, algo=4) == UNSUPPORTED     # E2M1 path: p, q <= 4 ...
    assert _gemm(lib, 64, 64, 128, 2, 6, algo=4) == UNSUPPORTED
    assert _gemm(lib, 64, 64, 32768, 4, 4, algo=4) == UNSUPPORTED   # ... and 4 K (2^p-1)(2^q-1) < 2^24
    assert b"" != lib.apmm_last_error()
    # 2^31 / (255 * 255) = 33025.5: K = 32768 = 64 * 512 fits, the next padded K (33280) does not
    assert _gemm(lib, 0, 4, 32768, 8, 8) == 0                       # M == 0: ok, nothing launched
    assert _gemm(lib, 4, 4, 32769, 8, 8) == OVERFLOW
    assert _gemm(lib, 4, 4, 40000, 8, 8) == OVERFLOW
    assert _gemm(lib, 64, 64, 128, 2, 2, algo=2) == INVALID         # an id no kernel of this build has
    assert _gemm(lib, 64, 64, 128, 4, 2, algo=7) == UNSUPPORTED     # plane kernels: activations of 1 or 2 bits
    assert _gemm(lib, 64, 64, 128, 5, 2, algo=8) == UNSUPPORTED     # K split across waves: p, q <= 4 like the E2M1 path
    assert _gemm(lib, 64, 64, 128, 2, 2, algo=6) == 4               # plane pairs to global memory: workspace missing
    assert lib.apmm_status_string(OVERFLOW) == b"result exceeds 32 bits"
    assert lib.apmm_pack_weights(None, 4, 128, 2, None, None) == INVALID
    assert lib.apmm_pack_activations(0x1000, 4, 128, 0, 0x2000, None) == INVALID
    assert lib.apmm_pack_weights(None, 0, 128, 2, None, None) == 0  # empty operand
    assert lib.apmm_unpack(None, 3, 128, 2, None, None) == INVALID


def test_new_entry_points_check_their_arguments(lib):
    """Fused quantise + pack, activation unpack and the grouped call reject bad arguments on the host."""
    from paper_2409_17870_amd.binding import ApmmProblem
    INVALID, OVERFLOW = 1, 3
    q = lib.apmm_quantize_pack_activations
    assert q(None, 4, 128, 2, 0x2000, 0x3000, None) == INVALID
    assert q(0x1000, 4, 128, 2, None, 0x3000, None) == INVALID
    assert q(0x1000, 4, 128, 2, 0x2000, None, None) == INVALID
    assert q(0x1000, 4, 0, 2, 0x2000, 0x3000, None) == INVALID
    assert q(0x1000, 4, 128, 9, 0x2000, 0x3000, None) == INVALID
    assert q(0x1001, 4, 128, 2, 0x2000, 0x3000, None) == INVALID       # binary16 data at an odd address
    assert q(0x1000, 0, 128, 2, 0x2000, 0x3000, None) == 0             # no rows: nothing to do
    assert lib.apmm_unpack_activations(None, 3, 128, 4, None, None) == INVALID
    fc = lib.apmm_gemm_from_codes
    fc.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 2 + [ctypes.c_void_p] * 7 + [ctypes.c_size_t, ctypes.c_void_p]
    assert fc(4, 8, 128, 2, 2, None, 0x2000, 0x3000, None, None, None, None, 0, None) == INVALID      # no codes
    assert fc(4, 8, 128, 2, 2, 0x1001, 0x2001, 0x3000, None, None, None, None, 0, None) == INVALID    # weights misaligned
    assert fc(4, 8, 128, 2, 2, 0x1001, 0x2000, None, None, None, None, None, 0, None) == INVALID      # no output
    assert fc(4, 8, 40000, 8, 8, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == OVERFLOW
    assert fc(0, 8, 128, 2, 2, None, None, None, None, None, None, None, 0, None) == 0                # no tokens
    # shapes outside the small-M kernels need a workspace for the packed activations: refused before any launch
    WORKSPACE = 4
    assert fc(65, 8, 128, 2, 2, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == WORKSPACE
    assert fc(17, 8, 128, 5, 2, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == WORKSPACE
    assert fc(33, 8, 128, 4, 2, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == WORKSPACE     # 4-bit activations: one launch up to 32 tokens
    assert fc(4, 8, 128, 2, 5, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == WORKSPACE
    assert fc(40, 8, 1 << 20, 2, 2, 0x1001, 0x2000, 0x3000, None, None, None, None, 0, None) == WORKSPACE   # K beyond the exact fp32 range
    need = lib.apmm_packed_activation_bytes(65, 128, 2)
    assert fc(65, 8, 128, 2, 2, 0x1001, 0x2000, 0x3000, None, None, None, 0x4000, need - 1, None) == WORKSPACE
    assert fc(65, 8, 128, 2, 2, 0x1001, 0x2000, 0x3000, None, None, None, 0x4004, need, None) == INVALID   # misaligned
    grouped = lib.apmm_gemm_grouped
    grouped.argtypes = [ctypes.c_int, ctypes.POINTER(ApmmProblem), ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                        ctypes.c_size_t, ctypes.c_void_p]
    assert grouped(0, None, 2, 2, None, 0, None) == 0
    assert grouped(2, None, 2, 2, None, 0, None) == INVALID
    assert grouped(-1, None, 2, 2, None, 0, None) == INVALID
    arr = (ApmmProblem * 2)()
    for pr in arr:
        pr.M, pr.N, pr.K, pr.a_packed, pr.w_packed, pr.c_i32 = 4, 8, 128, 0x1000, 0x2000, 0x3000
    arr[1].c_i32 = None                                                 # second entry asks for no output
    assert grouped(2, arr, 2, 2, None, 0, None) == INVALID              # nothing is launched for the first either
    arr[1].c_i32, arr[1].K = 0x3000, 40000
    assert grouped(2, arr, 8, 8, None, 0, None) == OVERFLOW
    arr[1].K = 128
    arr[0].a_codes, arr[0].a_packed, arr[0].M = 0x5001, None, 100      # unpacked codes: only shapes of the small-M kernels
    assert grouped(2, arr, 2, 2, None, 0, None) == 2
    big = (ApmmProblem * 300)()
    assert grouped(300, big, 2, 2, None, 0, None) == INVALID            # more entries than one call takes

