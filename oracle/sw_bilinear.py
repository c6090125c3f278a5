"""ctypes front end of the generic bilinear oracle (oracle/sw_bilinear_oracle.c).  TEST INFRASTRUCTURE ONLY."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsw_bilinear_oracle.so")
_lib = None
STRASSEN, CLASSICAL8 = 0, 1


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
        L.sw_bilinear_tables.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.sw_bilinear_tables.restype = ctypes.c_int
        L.sw_bilinear_get_counters.argtypes = [ctypes.POINTER(Counters)]
        _lib = L
    return _lib


def gemm(A, B, levels, scheme):
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    n = A.shape[0]
    C = np.empty_like(A)
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    rc = lib().sw_bilinear_gemm(n, p(A), p(B), p(C), int(levels), int(scheme))
    if rc != 0:
        raise RuntimeError(f"sw_bilinear_gemm failed with {rc}")
    return C


def tables(scheme):
    """(U, V, W) as integer arrays of shapes (q, 4), (q, 4), (4, q)."""
    buf = (ctypes.c_int * 96)()
    q = lib().sw_bilinear_tables(int(scheme), buf)
    v = np.array(buf[: 12 * q], dtype=np.int64)
    return v[: 4 * q].reshape(q, 4), v[4 * q: 8 * q].reshape(q, 4), v[8 * q:].reshape(4, q)


def reset_counters():
    lib().sw_bilinear_reset_counters()


def counters():
    c = Counters()
    lib().sw_bilinear_get_counters(ctypes.byref(c))
    return {n: int(getattr(c, n)) for n, _ in Counters._fields_}
