"""Seeded synthetic input matrices, shared by the tests of the CPU oracle and of the HIP path.

This module holds none of the method's arithmetic: it only defines what the
entries of A and B are.  Every entry is a pure function of (seed, matrix,
row, column), so any row, column or block can be regenerated anywhere without
holding the whole matrix:

    key   = 2*seed + which                    (which: 0 for A, 1 for B)
    k0    = mix(key + GAMMA)
    z     = mix(k0 + (idx + 1) * GAMMA)       idx = row * n + col, all mod 2^64
    mix   = the splitmix64 output function (Steele, Lea, Flood 2014):
            z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
            z *= 0x94D049BB133111EB; z ^= z >> 31
    u     = (z >> 11) * 2^-53                 in [0, 1)

distributions
    "uniform"    2u - 1                                   iid U[-1, 1)
    "rowscaled"  (2u - 1) * (1 + row / n)                 row-dependent magnitude
    "integer"    ((z >> 32) * 17 >> 32) - 8               iid integers in [-8, 8]
    "badscaled"  (2u - 1) * 2^(s(row) + g(col)) for A and (2u - 1) * 2^(-g(row) + t(col)) for B, with
                 s(i) = round(40 i / n) - 20, t(j) = 20 - round(40 j / n), g(k) = round(30 k / n) - 15:
                 rows of A, columns of B and the inner index span many binades (the case for the
                 diagonal scaling of Section 6.1); host only
    "normal"     sqrt(-2 ln u1) * cos(2 pi u2) with u1 = ((z1 >> 11) + 1) * 2^-53 and
                 u2 from counters 2*idx and 2*idx + 1     iid N(0, 1); host only

The first three use integer operations, one exact int->double conversion and
correctly rounded fp64 multiply/divide/add only, so the device fill kernel
(csrc/inputs_fill.hip, built into its own library, not part of the product)
produces the same bits; "normal" needs log and cos and is generated on the
host and uploaded.
"""
import ctypes
import os

import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

DISTS = ("uniform", "rowscaled", "integer", "normal", "badscaled")

# The five workloads of the build's baseline file (shape, depth, step order, distribution, seed).
CONFIGS = [
    dict(name="cfg1", n=256, levels=1, schedule="B", dist="uniform", seed=0),
    dict(name="cfg2", n=4096, levels=3, schedule="BBB", dist="uniform", seed=1),
    dict(name="cfg3", n=16384, levels=4, schedule="DBBB", dist="normal", seed=2),
    dict(name="cfg4", n=23520, levels=5, schedule="BDBDB", dist="rowscaled", seed=3),
    dict(name="cfg5", n=94080, levels=5, schedule=None, dist="uniform", seed=4),
]


def _mix(z):
    with np.errstate(over="ignore"):
        z = z ^ (z >> np.uint64(30))
        z = z * _M1
        z = z ^ (z >> np.uint64(27))
        z = z * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _bits(seed, which, idx):
    """64 random bits for every counter in idx (uint64 array)."""
    with np.errstate(over="ignore"):
        key = np.uint64(2 * int(seed) + int(which))
        k0 = _mix(np.asarray(key + GAMMA, dtype=np.uint64))
        return _mix(k0 + (idx + np.uint64(1)) * GAMMA)


def block(n, seed, which, dist, rows, cols):
    """Entries [rows x cols] of the n x n matrix `which` (0 = A, 1 = B) as float64.

    rows, cols: 1-D integer arrays (any order, repeats allowed)."""
    if dist not in DISTS:
        raise ValueError(f"unknown distribution {dist!r}")
    rows = np.asarray(rows, dtype=np.uint64).reshape(-1, 1)
    cols = np.asarray(cols, dtype=np.uint64).reshape(1, -1)
    with np.errstate(over="ignore"):
        idx = rows * np.uint64(n) + cols
        if dist == "normal":
            z1 = _bits(seed, which, idx * np.uint64(2))
            z2 = _bits(seed, which, idx * np.uint64(2) + np.uint64(1))
            u1 = ((z1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
            u2 = (z2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
            return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        z = _bits(seed, which, idx)
        if dist == "integer":
            k = ((z >> np.uint64(32)) * np.uint64(17)) >> np.uint64(32)
            return k.astype(np.float64) - 8.0
        u = (z >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        v = 2.0 * u - 1.0
        if dist == "rowscaled":
            v = v * (1.0 + rows.astype(np.float64) / float(n))
        if dist == "badscaled":
            r = rows.astype(np.float64)
            c = cols.astype(np.float64)
            g = lambda k: np.round(30.0 * k / n) - 15.0
            if which == 0:
                v = v * np.exp2((np.round(40.0 * r / n) - 20.0) + g(c))
            else:
                v = v * np.exp2(-g(r) + (20.0 - np.round(40.0 * c / n)))
        return v


def matrix(n, seed, which, dist, chunk_rows=1024):
    """The whole n x n matrix as a C-contiguous float64 array (generated in row chunks)."""
    out = np.empty((n, n), dtype=np.float64)
    cols = np.arange(n, dtype=np.uint64)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        out[r0:r1] = block(n, seed, which, dist, np.arange(r0, r1, dtype=np.uint64), cols)
    return out


def pair(cfg):
    """(A, B) on the host for one entry of CONFIGS (or any dict with n, seed, dist)."""
    return (matrix(cfg["n"], cfg["seed"], 0, cfg["dist"]),
            matrix(cfg["n"], cfg["seed"], 1, cfg["dist"]))


# ---- device fill (bit-identical for "uniform", "rowscaled", "integer") ------

_HERE = os.path.dirname(os.path.abspath(__file__))
FILL_LIB_PATH = os.path.join(_HERE, "libsw_inputs.so")
_fill_lib = None
_DIST_CODE = {"uniform": 0, "rowscaled": 1, "integer": 2}


def _fill():
    global _fill_lib
    if _fill_lib is None:
        if not os.path.exists(FILL_LIB_PATH):
            from . import build as _build          # a fresh checkout: compile once
            _build.build()
        if not os.path.exists(FILL_LIB_PATH):
            raise RuntimeError(f"{FILL_LIB_PATH} is not built; run __graft_entry__.build()")
        L = ctypes.CDLL(FILL_LIB_PATH)
        L.sw_inputs_fill.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                     ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.sw_inputs_fill.restype = ctypes.c_int
        _fill_lib = L
    return _fill_lib


def fill_device(t, n, seed, which, dist):
    """Fill the CUDA/HIP tensor t (n x n float64, row-major, dense) in place on torch's current stream."""
    import torch
    if dist not in _DIST_CODE:
        raise ValueError(f"{dist!r} has no device generator; generate on the host and upload")
    if t.dtype != torch.float64 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (n, n):
        raise ValueError("t must be a contiguous n x n float64 device tensor")
    stream = torch.cuda.current_stream(t.device).cuda_stream
    with torch.cuda.device(t.device):
        rc = _fill().sw_inputs_fill(t.data_ptr(), n, n, n, int(seed), int(which), _DIST_CODE[dist], stream)
    if rc != 0:
        raise RuntimeError(f"sw_inputs_fill failed with HIP error {rc}")
    return t


def device_pair(cfg, device="cuda:0"):
    """(A, B) as device tensors for one entry of CONFIGS; generated on the device when the
    distribution allows it, else on the host and uploaded."""
    import torch
    n = cfg["n"]
    out = []
    for which in (0, 1):
        if cfg["dist"] in _DIST_CODE:
            t = torch.empty((n, n), dtype=torch.float64, device=device)
            fill_device(t, n, cfg["seed"], which, cfg["dist"])
        else:
            t = torch.from_numpy(matrix(n, cfg["seed"], which, cfg["dist"])).to(device)
        out.append(t)
    return out[0], out[1]
