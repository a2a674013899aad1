"""CPU oracle for bipolar-INT arbitrary-precision GEMM (test infrastructure only).

Thin ctypes wrapper over ``apmm_oracle.c`` (plain C, int64 arithmetic).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product path never does, and this
package never imports the HIP binding.

Functions (paper passages in brackets):
  bipolar_value(code, nbits)            value of a code                 [Sec. 3.1, Eq. 1]
  gemm_i64(a_codes, w_codes, p, q)      C = A W^T on decoded values     [Sec. 3.2]
  gemm_planes_i64(a_codes, w_codes,..)  decomposition / 1-bit products /
                                        shift-add recovery              [Sec. 3.2]
  scale_f64(c, a_scale, w_scale)        double-precision scale epilogue
  quantize_rows(x_f16, p)               per-row symmetric quantisation of binary16
                                        features onto the bipolar-INT grid [Sec. 3.1]
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "apmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (OpenMP over output rows)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64, u8p = ctypes.c_int64, ctypes.POINTER(ctypes.c_uint8)
    i64p, u16p = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_uint16)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.oracle_bipolar_value.restype = i64
    lib.oracle_bipolar_value.argtypes = [ctypes.c_uint32, ctypes.c_int]
    lib.oracle_num_threads.restype = ctypes.c_int
    for name in ("oracle_gemm_i64", "oracle_gemm_planes_i64"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [i64, i64, i64, ctypes.c_int, ctypes.c_int, u8p, u8p, i64p]
    lib.oracle_half_bits_to_double.restype = ctypes.c_double
    lib.oracle_half_bits_to_double.argtypes = [ctypes.c_uint16]
    lib.oracle_scale_f64.restype = None
    lib.oracle_scale_f64.argtypes = [i64, i64, i64p, u16p, u16p, f64p]
    lib.oracle_float_to_half_bits.restype = ctypes.c_uint16
    lib.oracle_float_to_half_bits.argtypes = [ctypes.c_float]
    lib.oracle_quantize_rows.restype = None
    lib.oracle_quantize_rows.argtypes = [i64, i64, ctypes.c_int, u16p, u8p, u16p]
    lib.oracle_double_to_half_bits.restype = ctypes.c_uint16
    lib.oracle_double_to_half_bits.argtypes = [ctypes.c_double]
    _lib = lib
    return lib


def num_threads():
    return int(_load().oracle_num_threads())


def bipolar_value(code, nbits):
    return int(_load().oracle_bipolar_value(int(code), int(nbits)))


def _codes(x):
    x = np.ascontiguousarray(x, dtype=np.uint8)
    if x.ndim != 2:
        raise ValueError("codes must be a 2-D uint8 array (rows x K)")
    return x


def _gemm(fn_name, a_codes, w_codes, p, q):
    a, w = _codes(a_codes), _codes(w_codes)
    if a.shape[1] != w.shape[1]:
        raise ValueError("A and W must share K")
    M, K = a.shape
    N = w.shape[0]
    c = np.zeros((M, N), dtype=np.int64)
    if M == 0 or N == 0:
        return c
    u8p, i64p = ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_int64)
    rc = getattr(_load(), fn_name)(M, N, K, int(p), int(q),
                                   a.ctypes.data_as(u8p), w.ctypes.data_as(u8p),
                                   c.ctypes.data_as(i64p))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return c


def gemm_i64(a_codes, w_codes, p, q):
    """int64 C[m][n] = sum_k val_p(A[m][k]) * val_q(W[n][k])."""
    return _gemm("oracle_gemm_i64", a_codes, w_codes, p, q)


def gemm_planes_i64(a_codes, w_codes, p, q):
    """Same result through bit planes, 1-bit products and shift-add recovery."""
    return _gemm("oracle_gemm_planes_i64", a_codes, w_codes, p, q)


def gemm_i32(a_codes, w_codes, p, q):
    """The 32-bit output the paper states; raises if a value does not fit."""
    c = gemm_i64(a_codes, w_codes, p, q)
    if c.size and max(int(c.max()), -int(c.min())) > 2**31 - 1:
        raise OverflowError("result does not fit the 32-bit output")
    return c.astype(np.int32)


def half_bits_to_double(h):
    return float(_load().oracle_half_bits_to_double(int(h)))


def scale_f64(c, a_scale_bits=None, w_scale_bits=None):
    """F = C * a_scale[m] * w_scale[n] in double; scales are binary16 bit patterns (uint16)."""
    c = np.ascontiguousarray(c, dtype=np.int64)
    M, N = c.shape
    f = np.zeros((M, N), dtype=np.float64)
    if M == 0 or N == 0:
        return f
    u16p = ctypes.POINTER(ctypes.c_uint16)
    a = w = None
    ap = wp = ctypes.cast(None, u16p)
    if a_scale_bits is not None:
        a = np.ascontiguousarray(a_scale_bits, dtype=np.uint16)
        assert a.shape == (M,)
        ap = a.ctypes.data_as(u16p)
    if w_scale_bits is not None:
        w = np.ascontiguousarray(w_scale_bits, dtype=np.uint16)
        assert w.shape == (N,)
        wp = w.ctypes.data_as(u16p)
    _load().oracle_scale_f64(M, N, c.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                             ap, wp, f.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return f


def float_to_half_bits(f):
    return int(_load().oracle_float_to_half_bits(float(f)))


def double_to_half_bits(f):
    return int(_load().oracle_double_to_half_bits(float(f)))


def quantize_rows(x_f16, p):
    """(codes uint8 M x K, scale bit patterns uint16 M) of binary16 features x (M x K float16)."""
    x = np.ascontiguousarray(x_f16, dtype=np.float16)
    if x.ndim != 2:
        raise ValueError("x must be a 2-D float16 array (rows x K)")
    M, K = x.shape
    codes = np.zeros((M, K), dtype=np.uint8)
    scale = np.zeros((M,), dtype=np.uint16)
    if M and K:
        u8p, u16p = ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_uint16)
        _load().oracle_quantize_rows(M, K, int(p), x.view(np.uint16).ctypes.data_as(u16p),
                                     codes.ctypes.data_as(u8p), scale.ctypes.data_as(u16p))
    return codes, scale

