"""ctypes front end of the generic bilinear oracle (oracle/sw_bilinear_oracle.c).  TEST INFRASTRUCTURE ONLY."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsw_bilinear_oracle.so")
_lib = None
STRASSEN, CLASSICAL8, LADERMAN, CLASSICAL27 = 0, 1, 2, 3


class Counters(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("leaf_mul", "leaf_add", "block_add", "leaf_calls")]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            import importlib.util
            spec = importlib.util.spec_from_file_location("_sw_oracle_build", os.path.join(_HERE, "build.py"))
            mod = importlib.util.module_from_spec(spec)
            spec.loader.exec_module(mod)
            mod.build(force=True)
        L = ctypes.CDLL(_LIB_PATH)
        dp = ctypes.POINTER(ctypes.c_double)
        L.sw_bilinear_gemm.argtypes = [ctypes.c_int64, dp, dp, dp, ctypes.c_int, ctypes.c_int]
        L.sw_bilinear_gemm.restype = ctypes.c_int
        L.sw_bilinear_gemm_levels.argtypes = [ctypes.c_int64, dp, dp, dp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.sw_bilinear_gemm_levels.restype = ctypes.c_int
        L.sw_bilinear_tables.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.sw_bilinear_tables.restype = ctypes.c_int
        L.sw_bilinear_get_counters.argtypes = [ctypes.POINTER(Counters)]
        _lib = L
    return _lib


def gemm(A, B, levels, scheme):
    """C = A @ B by `levels` steps of one scheme (an int) or of one scheme per level (a sequence, top level first)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    n = A.shape[0]
    C = np.empty_like(A)
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    per_level = [int(scheme)] * int(levels) if np.isscalar(scheme) else [int(x) for x in scheme]
    if len(per_level) != int(levels):
        raise ValueError("one scheme per level")
    arr = (ctypes.c_int * max(1, len(per_level)))(*per_level)
    rc = lib().sw_bilinear_gemm_levels(n, p(A), p(B), p(C), int(levels), arr)
    if rc != 0:
        raise RuntimeError(f"sw_bilinear_gemm_levels failed with {rc}")
    return C


def tables(scheme):
    """(U, V, W, n0) with integer arrays of shapes (q, n0^2), (q, n0^2), (n0^2, q)."""
    buf = (ctypes.c_int * (3 * 27 * 9))()
    n0 = ctypes.c_int(0)
    q = lib().sw_bilinear_tables(int(scheme), buf, ctypes.byref(n0))
    if q < 0:
        raise ValueError("unknown scheme")
    b = n0.value ** 2
    v = np.array(buf[: 3 * q * b], dtype=np.int64)
    return v[: q * b].reshape(q, b), v[q * b: 2 * q * b].reshape(q, b), v[2 * q * b:].reshape(b, q), n0.value


def reset_counters():
    lib().sw_bilinear_reset_counters()


def counters():
    c = Counters()
    lib().sw_bilinear_get_counters(ctypes.byref(c))
    return {n: int(getattr(c, n)) for n, _ in Counters._fields_}
