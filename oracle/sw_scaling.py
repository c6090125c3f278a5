"""CPU oracle for the product with diagonal scaling (Section 6.1).  TEST INFRASTRUCTURE ONLY.

D1 C D3 = (D1 A D2)(D2^-1 B D3) with diagonal D1, D2, D3.  The paper leaves the choice of the D's open; the
reading taken (and listed in the design notes) is: powers of two, so that scaling is exact;
  outside  D1_ii = 2^-e(max_j |A_ij|), D3_jj = 2^-e(max_i |B_ij|)   with e(x) = floor(log2 x), e(0) = 0;
  inside   D2_kk = 2^round_half_away((e(max_j |B_kj| D3_jj) - e(max_i D1_ii |A_ik|)) / 2), 1 if either is 0.
Written with plain numpy; shares nothing with the HIP path.
"""
import numpy as np

import sw_oracle

OUTSIDE, INSIDE = 1, 2


def _exponent(m):
    e = np.zeros(m.shape, dtype=np.int64)
    ok = (m > 0) & np.isfinite(m)
    e[ok] = np.floor(np.log2(m[ok])).astype(np.int64)
    # floor(log2) can be off by one next to a power of two: fix it with exact comparisons
    e[ok] += (np.ldexp(1.0, e[ok] + 1) <= m[ok]).astype(np.int64)
    e[ok] -= (np.ldexp(1.0, e[ok]) > m[ok]).astype(np.int64)
    return e


def scales(A, B, scaling):
    """(d1, d2, d3) as float64 vectors of powers of two."""
    n = A.shape[0]
    d1 = np.ones(n)
    d2 = np.ones(n)
    d3 = np.ones(n)
    if scaling & OUTSIDE:
        d1 = np.ldexp(1.0, -_exponent(np.max(np.abs(A), axis=1)))
        d3 = np.ldexp(1.0, -_exponent(np.max(np.abs(B), axis=0)))
    if scaling & INSIDE:
        a = np.max(np.abs(A) * d1[:, None], axis=0)
        b = np.max(np.abs(B) * d3[None, :], axis=1)
        diff = _exponent(b) - _exponent(a)
        e = np.where(diff >= 0, (diff + 1) // 2, -((-diff + 1) // 2))
        e = np.where((a > 0) & (b > 0), e, 0)
        d2 = np.ldexp(1.0, e)
    return d1, d2, d3


def gemm_scaled(A, B, levels, scaling):
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    d1, d2, d3 = scales(A, B, scaling)
    As = d1[:, None] * A * d2[None, :]
    Bs = (1.0 / d2)[:, None] * B * d3[None, :]
    Cs = sw_oracle.gemm(As, Bs, levels)
    return (1.0 / d1)[:, None] * Cs * (1.0 / d3)[None, :]
