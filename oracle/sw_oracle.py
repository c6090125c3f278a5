"""ctypes front end of the CPU oracle (oracle/sw_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module; the product path never does.  It shares nothing with the HIP library.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsw_oracle.so")
_lib = None


class Counters(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int64) for name in
                ("leaf_mul", "leaf_add", "sw_add", "leaf_calls", "sw_steps", "mat_adds", "mat_mults")]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


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
        L.sw_oracle_gemm.argtypes = [ctypes.c_int64, dp, dp, dp, ctypes.c_int]
        L.sw_oracle_gemm.restype = ctypes.c_int
        L.sw_oracle_gemm_table.argtypes = [ctypes.c_int64, dp, dp, dp, ctypes.c_int, ctypes.c_int]
        L.sw_oracle_gemm_table.restype = ctypes.c_int
        L.sw_oracle_gemm_peel.argtypes = [ctypes.c_int64, dp, dp, dp, ctypes.c_int]
        L.sw_oracle_gemm_peel.restype = ctypes.c_int
        L.sw_oracle_naive.argtypes = [ctypes.c_int64, dp, dp, dp]
        L.sw_oracle_naive.restype = None
        L.sw_oracle_entry.argtypes = [ctypes.c_int64, dp, dp, ctypes.c_int64]
        L.sw_oracle_entry.restype = ctypes.c_double
        L.sw_oracle_row_strip.argtypes = [ctypes.c_int64, ctypes.c_int64, dp, dp, dp]
        L.sw_oracle_row_strip.restype = None
        L.sw_oracle_col_strip.argtypes = [ctypes.c_int64, ctypes.c_int64, dp, dp, dp]
        L.sw_oracle_col_strip.restype = None
        L.sw_oracle_reset_counters.argtypes = []
        L.sw_oracle_reset_counters.restype = None
        L.sw_oracle_get_counters.argtypes = [ctypes.POINTER(Counters)]
        L.sw_oracle_get_counters.restype = None
        L.sw_oracle_peak_words.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_char_p]
        L.sw_oracle_peak_words.restype = ctypes.c_int64
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _square(a, name):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError(f"{name} must be a square matrix")
    return a


def gemm(A, B, levels, table=0):
    """C = A @ B by `levels` Strassen-Winograd steps over a classical leaf (Appendix A).

    table=0: corrected tables; table=1: the tables exactly as printed (not a product)."""
    A = _square(A, "A")
    B = _square(B, "B")
    if A.shape != B.shape:
        raise ValueError("A and B differ in size")
    n = A.shape[0]
    C = np.empty_like(A)
    rc = lib().sw_oracle_gemm_table(n, _ptr(A), _ptr(B), _ptr(C), int(levels), int(table))
    if rc != 0:
        raise RuntimeError(f"sw_oracle_gemm_table failed with {rc}")
    return C


def gemm_peel(A, B, levels):
    """C = A @ B by `levels` Strassen-Winograd steps with the last row and column peeled off at every level whose size
    is odd (no padding); needs n >= 2^levels."""
    A = _square(A, "A")
    B = _square(B, "B")
    if A.shape != B.shape:
        raise ValueError("A and B differ in size")
    C = np.empty_like(A)
    rc = lib().sw_oracle_gemm_peel(A.shape[0], _ptr(A), _ptr(B), _ptr(C), int(levels))
    if rc != 0:
        raise RuntimeError(f"sw_oracle_gemm_peel failed with {rc}")
    return C


def naive(A, B):
    """C = A @ B by the definition C_ij = sum_k A_ik B_kj, k ascending (Algorithm 1, Ensure)."""
    A = _square(A, "A")
    B = _square(B, "B")
    C = np.empty_like(A)
    lib().sw_oracle_naive(A.shape[0], _ptr(A), _ptr(B), _ptr(C))
    return C


def entry(a_row, b_col):
    """One entry of A @ B from row i of A and column j of B, accumulated in long double."""
    a_row = np.ascontiguousarray(a_row, dtype=np.float64)
    b_col = np.ascontiguousarray(b_col, dtype=np.float64)
    if a_row.shape != b_col.shape or a_row.ndim != 1:
        raise ValueError("row and column must be 1-D and of equal length")
    return float(lib().sw_oracle_entry(a_row.shape[0], _ptr(a_row), _ptr(b_col), 1))


def row_strip(A_rows, B):
    """Rows of A @ B by the definition (k ascending): A_rows is r x n (chosen rows of A), B is n x n."""
    A_rows = np.ascontiguousarray(A_rows, dtype=np.float64)
    B = _square(B, "B")
    n = B.shape[0]
    if A_rows.ndim != 2 or A_rows.shape[1] != n:
        raise ValueError("A_rows must be r x n")
    C = np.empty_like(A_rows)
    lib().sw_oracle_row_strip(n, A_rows.shape[0], _ptr(A_rows), _ptr(B), _ptr(C))
    return C


def col_strip(A, B_cols):
    """Columns of A @ B by the definition (k ascending): A is n x n, B_cols is n x c (chosen columns of B)."""
    A = _square(A, "A")
    B_cols = np.ascontiguousarray(B_cols, dtype=np.float64)
    n = A.shape[0]
    if B_cols.ndim != 2 or B_cols.shape[0] != n:
        raise ValueError("B_cols must be n x c")
    C = np.empty_like(B_cols)
    lib().sw_oracle_col_strip(n, B_cols.shape[1], _ptr(A), _ptr(B_cols), _ptr(C))
    return C


def reset_counters():
    lib().sw_oracle_reset_counters()


def counters():
    c = Counters()
    lib().sw_oracle_get_counters(ctypes.byref(c))
    return c.as_dict()


def peak_words(n, levels, schedule):
    """Words of S/T/Q storage beyond A, B, C that a traversal holds at its peak
    (Sections 3.3.1, 3.4.1), found by walking the tree."""
    r = lib().sw_oracle_peak_words(int(n), int(levels), schedule.encode())
    if r < 0:
        raise ValueError("bad n / levels / schedule")
    return int(r)
