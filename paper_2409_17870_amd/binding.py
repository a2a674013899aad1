"""ctypes binding of libapmm.so (C ABI in include/apmm.h).

Argument marshalling only: every step of the path (pack, GEMM, recovery, epilogue) runs
in the library's HIP kernels.  PyTorch supplies device memory and the stream.  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch  # imported before the library so that both share one HIP runtime (same soname)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libapmm.so")

ALGO_AUTO, ALGO_VALU_POPCOUNT, ALGO_DECODE, ALGO_MFMA_FP4, ALGO_DECODE_VALU = 0, 1, 3, 4, 5
ALGO_PLANE_PAIRS_GLOBAL, ALGO_PLANES_REGISTERS, ALGO_MFMA_KSPLIT = 6, 7, 8

EXPORTS = [
    "apmm_packed_bytes", "apmm_packed_activation_bytes", "apmm_workspace_bytes", "apmm_pack_weights", "apmm_pack_activations",
    "apmm_quantize_pack_activations", "apmm_unpack", "apmm_unpack_activations", "apmm_gemm", "apmm_gemm_ex", "apmm_gemm_from_codes", "apmm_gemm_from_codes_noalloc", "apmm_gemm_grouped",
    "apmm_time_next_gemm", "apmm_last_gemm_kernel", "apmm_status_string", "apmm_last_error", "apmm_version",
]



class ApmmProblem(ctypes.Structure):
    """struct apmm_problem of include/apmm.h"""
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("a_packed", ctypes.c_void_p), ("w_packed", ctypes.c_void_p),
                ("c_i32", ctypes.c_void_p), ("c_f16", ctypes.c_void_p),
                ("w_scale", ctypes.c_void_p), ("a_scale", ctypes.c_void_p), ("a_codes", ctypes.c_void_p)]


_lib = None


class ApmmError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("apmm status %d: %s" % (status, text))
        self.status = status


def load():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.apmm_packed_bytes.restype = ctypes.c_size_t
    lib.apmm_packed_bytes.argtypes = [i64, i64, ci]
    lib.apmm_packed_activation_bytes.restype = ctypes.c_size_t
    lib.apmm_packed_activation_bytes.argtypes = [i64, i64, ci]
    lib.apmm_workspace_bytes.restype = ctypes.c_size_t
    lib.apmm_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    for name in ("apmm_pack_weights", "apmm_pack_activations"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.apmm_quantize_pack_activations.restype = ci
    lib.apmm_quantize_pack_activations.argtypes = [vp, i64, i64, ci, vp, vp, vp]
    for name in ("apmm_unpack", "apmm_unpack_activations"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, i64, i64, ci, vp, vp]
    gemm_args = [i64, i64, i64, ci, ci, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.apmm_gemm.restype = ci
    lib.apmm_gemm.argtypes = gemm_args
    lib.apmm_gemm_ex.restype = ci
    lib.apmm_gemm_ex.argtypes = gemm_args + [ci]
    lib.apmm_gemm_from_codes.restype = ci
    lib.apmm_gemm_from_codes.argtypes = gemm_args
    lib.apmm_gemm_from_codes_noalloc.restype = ci
    lib.apmm_gemm_from_codes_noalloc.argtypes = [i64, i64, i64, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.apmm_gemm_grouped.restype = ci
    lib.apmm_gemm_grouped.argtypes = [ci, ctypes.POINTER(ApmmProblem), ci, ci, vp, ctypes.c_size_t, vp]
    lib.apmm_time_next_gemm.restype = ci
    lib.apmm_time_next_gemm.argtypes = [vp, vp]
    lib.apmm_last_gemm_kernel.restype = ctypes.c_char_p
    lib.apmm_last_gemm_kernel.argtypes = []
    lib.apmm_status_string.restype = ctypes.c_char_p
    lib.apmm_status_string.argtypes = [ci]
    lib.apmm_last_error.restype = ctypes.c_char_p
    lib.apmm_last_error.argtypes = []
    lib.apmm_version.restype = ci
    lib.apmm_version.argtypes = []
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        lib = load()
        text = lib.apmm_last_error().decode() or lib.apmm_status_string(status).decode()
        raise ApmmError(status, text)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(None)


def _dev_u8(t, what):
    if t.dtype != torch.uint8 or not t.is_cuda or not t.is_contiguous() or t.dim() != 2:
        raise ValueError("%s must be a contiguous 2-D uint8 CUDA tensor" % what)


def apmm_packed_bytes(rows, K, bits):
    return int(load().apmm_packed_bytes(rows, K, bits))


def apmm_packed_activation_bytes(M, K, p):
    return int(load().apmm_packed_activation_bytes(M, K, p))


def apmm_workspace_bytes(M, N, K, p, q):
    return int(load().apmm_workspace_bytes(M, N, K, p, q))


def _pack(fn_name, codes, bits, out):
    _dev_u8(codes, "codes")
    rows, K = codes.shape
    nbytes = (apmm_packed_activation_bytes if fn_name == "apmm_pack_activations" else apmm_packed_bytes)(rows, K, bits)
    if out is None:
        out = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=codes.device)
    elif out.numel() * out.element_size() < nbytes:
        raise ValueError("packed buffer too small")
    _check(getattr(load(), fn_name)(_ptr(codes), rows, K, bits, _ptr(out), _stream()))
    return out


def apmm_pack_weights(w_codes, q, out=None):
    """N x K uint8 weight codes -> opaque packed buffer (uint8 tensor)."""
    return _pack("apmm_pack_weights", w_codes, q, out)


def apmm_pack_activations(a_codes, p, out=None):
    """M x K uint8 activation codes -> opaque packed buffer (uint8 tensor)."""
    return _pack("apmm_pack_activations", a_codes, p, out)


def apmm_quantize_pack_activations(x_f16, p, out=None, scale_out=None):
    """M x K float16 activations -> (opaque packed buffer, float16 per-token scales)."""
    if x_f16.dtype != torch.float16 or not x_f16.is_cuda or not x_f16.is_contiguous() or x_f16.dim() != 2:
        raise ValueError("x must be a contiguous 2-D float16 CUDA tensor")
    M, K = x_f16.shape
    nbytes = apmm_packed_activation_bytes(M, K, p)
    if out is None:
        out = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=x_f16.device)
    elif out.numel() * out.element_size() < nbytes:
        raise ValueError("packed buffer too small")
    if scale_out is None:
        scale_out = torch.empty(M, dtype=torch.float16, device=x_f16.device)
    elif scale_out.dtype != torch.float16 or scale_out.numel() < M:
        raise ValueError("scale_out must hold M float16 values")
    _check(load().apmm_quantize_pack_activations(_ptr(x_f16), M, K, p, _ptr(out), _ptr(scale_out), _stream()))
    return out, scale_out


def apmm_unpack(packed, rows, K, bits):
    """Packed weights -> N x K uint8 codes."""
    codes = torch.empty((rows, K), dtype=torch.uint8, device=packed.device)
    _check(load().apmm_unpack(_ptr(packed), rows, K, bits, _ptr(codes), _stream()))
    return codes


def apmm_unpack_activations(a_packed, M, K, p):
    """Packed activations -> M x K uint8 codes."""
    codes = torch.empty((M, K), dtype=torch.uint8, device=a_packed.device)
    _check(load().apmm_unpack_activations(_ptr(a_packed), M, K, p, _ptr(codes), _stream()))
    return codes


def apmm_gemm(M, N, K, p, q, a_packed, w_packed, want_i32=True, want_f16=False, w_scale=None, a_scale=None,
              c_i32=None, c_f16=None, workspace=None, algo=ALGO_AUTO):
    """C = A W^T on packed operands.  Returns (c_i32 or None, c_f16 or None).

    w_scale / a_scale are float16 CUDA vectors of length N / M (or None).  c_i32 / c_f16 may be
    preallocated outputs (int32 / float16, M x N).
    """
    dev = a_packed.device
    if want_i32 and c_i32 is None:
        c_i32 = torch.empty((M, N), dtype=torch.int32, device=dev)
    if want_f16 and c_f16 is None:
        c_f16 = torch.empty((M, N), dtype=torch.float16, device=dev)
    for s, n, what in ((w_scale, N, "w_scale"), (a_scale, M, "a_scale")):
        if s is not None and (s.dtype != torch.float16 or s.numel() != n or not s.is_cuda
                              or not s.is_contiguous()):
            raise ValueError("%s must be a contiguous float16 CUDA vector of the right length" % what)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().apmm_gemm_ex(M, N, K, p, q, _ptr(a_packed), _ptr(w_packed), _ptr(c_i32), _ptr(c_f16),
                               _ptr(w_scale), _ptr(a_scale), _ptr(workspace), ws_bytes, _stream(), algo))
    return c_i32, c_f16


def apmm_gemm_from_codes(a_codes, N, p, q, w_packed, want_i32=True, want_f16=False, w_scale=None, a_scale=None,
                         c_i32=None, c_f16=None, workspace=None):
    """C = A W^T straight from the M x K uint8 activation codes: one launch for a few tokens, else packing
    into `workspace` (uint8 tensor of apmm_packed_activation_bytes(M, K, p) bytes) followed by the GEMM."""
    _dev_u8(a_codes, "a_codes")
    M, K = a_codes.shape
    dev = a_codes.device
    if want_i32 and c_i32 is None:
        c_i32 = torch.empty((M, N), dtype=torch.int32, device=dev)
    if want_f16 and c_f16 is None:
        c_f16 = torch.empty((M, N), dtype=torch.float16, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().apmm_gemm_from_codes(M, N, K, p, q, _ptr(a_codes), _ptr(w_packed), _ptr(c_i32), _ptr(c_f16),
                                       _ptr(w_scale), _ptr(a_scale), _ptr(workspace), ws_bytes, _stream()))
    return c_i32, c_f16


NOALLOC_MAX_PACKED_BYTES = 8 << 20  # APMM_NOALLOC_MAX_PACKED_BYTES of include/apmm.h


def apmm_gemm_from_codes_noalloc(a_codes, N, p, q, w_packed, c_i32=None, c_f16=None, w_scale=None, a_scale=None):
    """apmm_gemm_from_codes with the packed activations in the library's built-in buffer.  The call itself
    allocates nothing: the outputs are the caller's preallocated tensors."""
    _dev_u8(a_codes, "a_codes")
    M, K = a_codes.shape
    _check(load().apmm_gemm_from_codes_noalloc(M, N, K, p, q, _ptr(a_codes), _ptr(w_packed), _ptr(c_i32), _ptr(c_f16),
                                               _ptr(w_scale), _ptr(a_scale), _stream()))
    return c_i32, c_f16


def apmm_version():
    return int(load().apmm_version())


def apmm_gemm_grouped(problems, p, q):
    """Several GEMMs of equal p, q with as few launches as possible.

    problems: list of dicts with keys M, N, K, w_packed, a_packed or a_codes (unpacked uint8 codes, small-M
    shapes only) and optionally c_i32, c_f16 (output tensors), w_scale, a_scale.  Outputs must be preallocated
    by the caller.
    """
    arr = (ApmmProblem * max(len(problems), 1))()
    for i, pr in enumerate(problems):
        arr[i].M, arr[i].N, arr[i].K = pr["M"], pr["N"], pr["K"]
        for key in ("a_packed", "w_packed", "c_i32", "c_f16", "w_scale", "a_scale", "a_codes"):
            t = pr.get(key)
            setattr(arr[i], key, t.data_ptr() if t is not None else None)
    _check(load().apmm_gemm_grouped(len(problems), arr, p, q, None, 0, _stream()))


def apmm_last_gemm_kernel():
    """Name of the GEMM kernel the last GEMM call of this thread launched."""
    return load().apmm_last_gemm_kernel().decode()


def apmm_time_next_gemm(start_event, stop_event):
    """Attach two torch.cuda.Event (created with enable_timing=True and recorded once, so that their
    handles exist) to the kernel dispatch of the next large-tile MFMA GEMM call of this thread."""
    _check(load().apmm_time_next_gemm(ctypes.c_void_p(start_event.cuda_event), ctypes.c_void_p(stop_event.cuda_event)))

