"""Thin ctypes binding of libsw_gemm.so: the same names as the C ABI (include/sw_gemm.h), argument
marshalling only.  Tensors are torch CUDA (HIP) tensors used for their device memory; every step of the
path runs in the library's kernels.  There is no CPU fallback: a missing library raises."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SW_GEMM_LIB") or os.path.join(_HERE, "libsw_gemm.so")   # override: a library built elsewhere

SW_OK, SW_EINVAL, SW_ENOMEM, SW_EHIP = 0, -1, -2, -3
SW_MAX_LEVELS = 16
CLASS_NAMES = ("pre_add", "post_add", "leaf_gemm", "dfs_add", "pad", "peel", "scale", "blas")
SW_SCALE_OUTSIDE, SW_SCALE_INSIDE = 1, 2
SW_ODD_PAD, SW_ODD_PEEL, SW_ODD_PEEL_LEVELS = 0, 1, 2

EXPORTS = ("sw_gemm", "sw_gemm_ex", "sw_gemm_scaled", "sw_plan_memory_scaled", "sw_plan_memory", "sw_plan_workspace", "sw_plan_schedule", "sw_model_words", "sw_lm_dfs_steps",
           "sw_flop_count", "sw_set_workspace", "sw_set_stream", "sw_set_odd_mode", "sw_set_overlap", "sw_gemm_classical", "sw_last_error", "sw_pre_add", "sw_post_add",
           "sw_pre_add2", "sw_post_add2", "sw_leaf_gemm", "sw_pad_copy", "sw_profile_enable", "sw_profile_read",
           "sw_gemm_bilinear", "sw_plan_memory_bilinear", "sw_flop_count_bilinear", "sw_dgemm", "sw_plan_memory_dgemm",
           "sw_plan_levels", "sw_model_seconds", "sw_gemm_rect", "sw_plan_memory_rect", "sw_trace_gemm", "sw_gemm_static", "sw_gemm_bilinear_levels", "sw_plan_memory_bilinear_levels", "sw_model_seconds_order")


class SwError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"sw_gemm library error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Load libsw_gemm.so.  If nothing is built yet (a fresh checkout) it is compiled once with hipcc; if that
    fails, or a library named by SW_GEMM_LIB is missing, this raises: there is no other implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if os.environ.get("SW_GEMM_LIB"):
            raise RuntimeError(f"{LIB_PATH} (SW_GEMM_LIB) does not exist")
        from . import build as _build
        _build.build()
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing and could not be built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    i64, vp, cp, ci, dbl = ctypes.c_int64, ctypes.c_void_p, ctypes.c_char_p, ctypes.c_int, ctypes.c_double
    sig = {
        "sw_gemm": (ci, [i64, vp, vp, vp, ci, cp]),
        "sw_gemm_ex": (ci, [i64, vp, i64, vp, i64, vp, i64, ci, cp, vp, i64, vp]),
        "sw_gemm_static": (ci, [i64, vp, i64, vp, i64, vp, i64, ci, cp, vp]),
        "sw_plan_memory": (i64, [i64, ci, cp]),
        "sw_gemm_scaled": (ci, [i64, vp, vp, vp, ci, cp, ci]),
        "sw_plan_memory_scaled": (i64, [i64, ci, cp]),
        "sw_gemm_rect": (ci, [i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, cp, vp, i64, vp]),
        "sw_plan_memory_rect": (i64, [i64, i64, i64, ci, cp]),
        "sw_trace_gemm": (i64, [i64, i64, i64, i64, i64, i64, ci, cp, i64, ci, ci, i64, ctypes.POINTER(i64), i64]),
        "sw_dgemm": (ci, [ci, ci, i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, ci, cp]),
        "sw_plan_memory_dgemm": (i64, [ci, ci, i64, i64, i64, ci, cp]),
        "sw_plan_levels": (ci, [i64, i64]),
        "sw_model_seconds": (dbl, [i64, ci, i64]),
        "sw_model_seconds_order": (dbl, [i64, ci, cp, i64, ci]),
        "sw_gemm_bilinear": (ci, [i64, vp, vp, vp, ci, cp, ci]),
        "sw_plan_memory_bilinear": (i64, [i64, ci, cp, ci]),
        "sw_flop_count_bilinear": (dbl, [i64, ci, ci]),
        "sw_gemm_bilinear_levels": (ci, [i64, vp, vp, vp, ci, cp, ctypes.POINTER(ci)]),
        "sw_plan_memory_bilinear_levels": (i64, [i64, ci, cp, ctypes.POINTER(ci)]),
        "sw_plan_workspace": (i64, [i64, ci, cp, i64]),
        "sw_plan_schedule": (ci, [i64, ci, i64, ctypes.c_char_p]),
        "sw_model_words": (i64, [i64, ci, cp]),
        "sw_lm_dfs_steps": (ci, [dbl, dbl, dbl]),
        "sw_flop_count": (dbl, [i64, ci]),
        "sw_set_workspace": (ci, [vp, i64]),
        "sw_set_stream": (ci, [vp]),
        "sw_set_odd_mode": (ci, [ci]),
        "sw_set_overlap": (ci, [ci]),
        "sw_gemm_classical": (ci, [i64, i64, i64, vp, i64, vp, i64, vp, i64, ci, vp]),
        "sw_last_error": (cp, []),
        "sw_pre_add": (ci, [ci, vp, i64, i64, i64, i64, vp, i64, i64, vp]),
        "sw_post_add": (ci, [vp, i64, i64, i64, i64, vp, i64, i64, vp]),
        "sw_pre_add2": (ci, [ci, vp, i64, i64, i64, i64, vp, i64, i64, vp]),
        "sw_post_add2": (ci, [vp, i64, i64, i64, i64, vp, i64, i64, vp]),
        "sw_leaf_gemm": (ci, [i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, vp]),
        "sw_pad_copy": (ci, [vp, i64, i64, i64, vp, i64, i64, i64, vp]),
        "sw_profile_enable": (ci, [ci]),
        "sw_profile_read": (ci, [ctypes.POINTER(dbl), ctypes.POINTER(i64), ctypes.POINTER(dbl)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _check(rc):
    if rc < 0:
        raise SwError(int(rc), lib().sw_last_error().decode())
    return rc


def _sched(s):
    return None if s is None else s.encode()


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _stream(t):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _f64_cuda(t, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float64):
        raise TypeError(f"{name} must be a float64 tensor on the GPU")


# ---- host-only calls ----------------------------------------------------------------------------------------

def sw_plan_memory(n, levels, schedule=None):
    return _check(lib().sw_plan_memory(n, levels, _sched(schedule)))


def sw_plan_workspace(n, levels, schedule, budget_bytes):
    return _check(lib().sw_plan_workspace(n, levels, _sched(schedule), budget_bytes))


def sw_plan_schedule(n, levels, budget_bytes):
    buf = ctypes.create_string_buffer(SW_MAX_LEVELS + 1)
    _check(lib().sw_plan_schedule(n, levels, budget_bytes, buf))
    return buf.value.decode()


def sw_model_words(n, levels, schedule):
    return _check(lib().sw_model_words(n, levels, _sched(schedule)))


def sw_lm_dfs_steps(n, P, M_words):
    return _check(lib().sw_lm_dfs_steps(float(n), float(P), float(M_words)))


def sw_flop_count(n, levels):
    v = lib().sw_flop_count(n, levels)
    if v < 0:
        raise SwError(SW_EINVAL, "n must be a multiple of 2^levels")
    return v


def sw_last_error():
    return lib().sw_last_error().decode()


def sw_trace_gemm(M, N, K, lda, ldb, ldc, levels, schedule, workspace_bytes, overlap=1, odd_mode=SW_ODD_PAD, withhold=-1):
    """The record of a launch-free run of sw_gemm_rect as a numpy int64 array (format: include/sw_gemm.h)."""
    import numpy as np
    args = (M, N, K, lda, ldb, ldc, levels, _sched(schedule), workspace_bytes, int(overlap), odd_mode, withhold)
    words = _check(lib().sw_trace_gemm(*args, None, 0))
    log = np.empty(max(words, 1), dtype=np.int64)
    got = _check(lib().sw_trace_gemm(*args, log.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), words))
    assert got == words
    return log[:words]


# ---- device calls ----------------------------------------------------------------------------------------------

def sw_set_workspace(ws):
    """ws: a uint8/any CUDA tensor the caller keeps alive, or None to clear."""
    if ws is None:
        return _check(lib().sw_set_workspace(None, 0))
    return _check(lib().sw_set_workspace(_ptr(ws), ws.numel() * ws.element_size()))


def sw_set_stream(stream_handle):
    return _check(lib().sw_set_stream(ctypes.c_void_p(stream_handle)))


def sw_set_overlap(on):
    """False/0: one stream; True/1: three streams, leaf-side addition kernels sized to their work; k > 1: capped at k workgroups."""
    return _check(lib().sw_set_overlap(int(on)))


def sw_set_odd_mode(mode):
    return _check(lib().sw_set_odd_mode(mode))


def sw_gemm_classical(M, N, K, A, lda, B, ldb, C, ldc, accumulate=False):
    return _check(lib().sw_gemm_classical(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, 1 if accumulate else 0,
                                          _stream(C)))


def sw_gemm(n, A, B, C, levels, schedule=None):
    """C = A @ B through the library state set by sw_set_workspace / sw_set_stream."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
        if not t.is_contiguous() or tuple(t.shape) != (n, n):
            raise ValueError(f"{name} must be a contiguous {n} x {n} tensor")
    return _check(lib().sw_gemm(n, _ptr(A), _ptr(B), _ptr(C), levels, _sched(schedule)))


def sw_gemm_scaled(n, A, B, C, levels, schedule, scaling):
    """C = A @ B with diagonal scaling (Section 6.1) through the library state (workspace, stream)."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
        if not t.is_contiguous() or tuple(t.shape) != (n, n):
            raise ValueError(f"{name} must be a contiguous {n} x {n} tensor")
    return _check(lib().sw_gemm_scaled(n, _ptr(A), _ptr(B), _ptr(C), levels, _sched(schedule), scaling))


def sw_plan_memory_scaled(n, levels, schedule=None):
    return _check(lib().sw_plan_memory_scaled(n, levels, _sched(schedule)))


def sw_gemm_rect(M, N, K, A, lda, B, ldb, C, ldc, levels, schedule, workspace, stream_handle=None):
    """C (M x N) = A (M x K) @ B (K x N) by the same recursion on rectangular operands."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
    ws_ptr = None if workspace is None else _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = _stream(C) if stream_handle is None else ctypes.c_void_p(stream_handle)
    return _check(lib().sw_gemm_rect(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, levels, _sched(schedule), ws_ptr, ws_bytes, st))


def sw_plan_memory_rect(M, N, K, levels, schedule=None):
    return _check(lib().sw_plan_memory_rect(M, N, K, levels, _sched(schedule)))


def sw_dgemm(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, levels, schedule=None):
    """C <- alpha * op(A) @ op(B) + beta * C on row-major CUDA float64 tensors, through the library state."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        if t is not None:
            _f64_cuda(t, name)
    p = lambda t: None if t is None else _ptr(t)
    return _check(lib().sw_dgemm(int(bool(transa)), int(bool(transb)), M, N, K, float(alpha), p(A), lda, p(B), ldb,
                                 float(beta), p(C), ldc, levels, _sched(schedule)))


def sw_plan_memory_dgemm(transa, transb, M, N, K, levels, schedule=None):
    return _check(lib().sw_plan_memory_dgemm(int(bool(transa)), int(bool(transb)), M, N, K, levels, _sched(schedule)))


def sw_plan_levels(n, budget_bytes):
    return _check(lib().sw_plan_levels(n, int(budget_bytes)))


def sw_model_seconds(n, levels, budget_bytes):
    return lib().sw_model_seconds(n, levels, int(budget_bytes))


def sw_model_seconds_order(n, levels, schedule, budget_bytes, overlap=1):
    return lib().sw_model_seconds_order(n, levels, _sched(schedule), int(budget_bytes), int(overlap))


SW_SCHEME_WINOGRAD, SW_SCHEME_STRASSEN, SW_SCHEME_CLASSICAL, SW_SCHEME_LADERMAN, SW_SCHEME_CLASSICAL3 = 0, 1, 2, 3, 4
SCHEME_BASE = {SW_SCHEME_WINOGRAD: 2, SW_SCHEME_STRASSEN: 2, SW_SCHEME_CLASSICAL: 2, SW_SCHEME_LADERMAN: 3, SW_SCHEME_CLASSICAL3: 3}
SCHEME_PRODUCTS = {SW_SCHEME_WINOGRAD: 7, SW_SCHEME_STRASSEN: 7, SW_SCHEME_CLASSICAL: 8, SW_SCHEME_LADERMAN: 23, SW_SCHEME_CLASSICAL3: 27}


def _schemes(schemes):
    return (ctypes.c_int * max(1, len(schemes)))(*[int(x) for x in schemes])


def sw_gemm_bilinear_levels(n, A, B, C, schedule, schemes):
    """C = A @ B with one block scheme per level (top level first) through the library state."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
        if not t.is_contiguous() or tuple(t.shape) != (n, n):
            raise ValueError(f"{name} must be a contiguous {n} x {n} tensor")
    return _check(lib().sw_gemm_bilinear_levels(n, _ptr(A), _ptr(B), _ptr(C), len(schemes), _sched(schedule), _schemes(schemes)))


def sw_plan_memory_bilinear_levels(n, schedule, schemes):
    return _check(lib().sw_plan_memory_bilinear_levels(n, len(schemes), _sched(schedule), _schemes(schemes)))


def sw_gemm_bilinear(n, A, B, C, levels, schedule, scheme):
    """C = A @ B by the recursion of another 2 x 2 block scheme (Section 6.6) through the library state."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
        if not t.is_contiguous() or tuple(t.shape) != (n, n):
            raise ValueError(f"{name} must be a contiguous {n} x {n} tensor")
    return _check(lib().sw_gemm_bilinear(n, _ptr(A), _ptr(B), _ptr(C), levels, _sched(schedule), scheme))


def sw_plan_memory_bilinear(n, levels, schedule, scheme):
    return _check(lib().sw_plan_memory_bilinear(n, levels, _sched(schedule), scheme))


def sw_flop_count_bilinear(n, levels, scheme):
    return lib().sw_flop_count_bilinear(n, levels, scheme)


def sw_gemm_ex(n, A, lda, B, ldb, C, ldc, levels, schedule, workspace, stream_handle=None):
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
    ws_ptr = None if workspace is None else _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = _stream(C) if stream_handle is None else ctypes.c_void_p(stream_handle)
    return _check(lib().sw_gemm_ex(n, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, levels, _sched(schedule),
                                   ws_ptr, ws_bytes, st))


SW_STATIC_SCRATCH_BYTES = 128 * 1024 * 1024


def sw_gemm_static(n, A, lda, B, ldb, C, ldc, levels, schedule, stream_handle=None):
    """sw_gemm_ex on the library's own static scratch: allocates nothing (the caller passes C)."""
    for t, name in ((A, "A"), (B, "B"), (C, "C")):
        _f64_cuda(t, name)
    st = _stream(C) if stream_handle is None else ctypes.c_void_p(stream_handle)
    return _check(lib().sw_gemm_static(n, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, levels, _sched(schedule), st))


def sw_pre_add(side, parent, parent_ld, parent_stride, live, h, child, child_ld, child_stride):
    return _check(lib().sw_pre_add(side, _ptr(parent), parent_ld, parent_stride, live, h, _ptr(child), child_ld,
                                   child_stride, _stream(child)))


def sw_post_add(Q, q_ld, q_stride, live, h, parent, parent_ld, parent_stride):
    return _check(lib().sw_post_add(_ptr(Q), q_ld, q_stride, live, h, _ptr(parent), parent_ld, parent_stride,
                                    _stream(parent)))


def sw_pre_add2(side, parent, parent_ld, parent_stride, live, m, child, child_ld, child_stride):
    return _check(lib().sw_pre_add2(side, _ptr(parent), parent_ld, parent_stride, live, m, _ptr(child), child_ld,
                                    child_stride, _stream(child)))


def sw_post_add2(Q, q_ld, q_stride, live, m, parent, parent_ld, parent_stride):
    return _check(lib().sw_post_add2(_ptr(Q), q_ld, q_stride, live, m, _ptr(parent), parent_ld, parent_stride,
                                     _stream(parent)))


def sw_leaf_gemm(m, batch, A, lda, stride_a, B, ldb, stride_b, C, ldc, stride_c):
    return _check(lib().sw_leaf_gemm(m, batch, _ptr(A), lda, stride_a, _ptr(B), ldb, stride_b, _ptr(C), ldc,
                                     stride_c, _stream(C)))


def sw_pad_copy(src, src_ld, rows, cols, dst, dst_ld, prows, pcols):
    return _check(lib().sw_pad_copy(_ptr(src), src_ld, rows, cols, _ptr(dst), dst_ld, prows, pcols, _stream(dst)))


def sw_profile_enable(on):
    return _check(lib().sw_profile_enable(1 if on else 0))


def sw_profile_read():
    """-> {class name: dict(ms=..., launches=..., work=...)}; work is bytes for add kernels, flops for leaf_gemm."""
    n = len(CLASS_NAMES)
    ms = (ctypes.c_double * n)()
    launches = (ctypes.c_int64 * n)()
    work = (ctypes.c_double * n)()
    _check(lib().sw_profile_read(ms, launches, work))
    return {CLASS_NAMES[i]: dict(ms=ms[i], launches=int(launches[i]), work=work[i]) for i in range(n)}


# ---- convenience on top of the ABI (allocation of the workspace with torch; no arithmetic) ---------------------

def matmul(A, B, levels=None, schedule=None, workspace=None):
    """C = A @ B for square float64 CUDA tensors.  Allocates C and, if none is given, a workspace: of exactly
    sw_plan_memory bytes for a given step order, else what the planner can use of 80 % of the free device
    memory.  levels None: the depth sw_plan_levels picks for that budget."""
    import torch
    _f64_cuda(A, "A")
    _f64_cuda(B, "B")
    n = A.shape[0]
    A = A.contiguous()
    B = B.contiguous()
    C = torch.empty_like(A)
    if workspace is None:
        free, _ = torch.cuda.mem_get_info(A.device)
        budget = int(free * 0.8)
        if levels is None:
            levels = sw_plan_levels(n, budget)
            schedule = None
        if schedule is None:
            schedule = sw_plan_schedule(n, levels, budget)
            need = sw_plan_workspace(n, levels, schedule, budget)
        else:
            need = sw_plan_memory(n, levels, schedule)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=A.device)
    elif levels is None:
        levels, schedule = -1, None
    with torch.cuda.device(A.device):
        sw_gemm_ex(n, A, n, B, n, C, n, levels, schedule, workspace)
    return C
