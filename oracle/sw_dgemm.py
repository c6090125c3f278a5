"""Oracle of the general product C <- alpha * op(A) * op(B) + beta * C, op(X) = X or its transpose.
TEST INFRASTRUCTURE ONLY.

This is the textbook definition written out entry by entry: c_ij <- alpha * sum_k op(A)_ik op(B)_kj + beta * c_ij,
the sum taken in extended precision (numpy longdouble) with k ascending and rounded to fp64 once at the end.
The fast algorithms are drop-in replacements for this operation (Section 1 and Section 6: the same product,
computed with fewer multiplications); what they may differ by is bounded by the norm-wise bound of Section 6.1.
By the usual convention beta = 0 means C is not read (a NaN in it does not propagate) and alpha = 0 means
A and B are not read.  Shares no code with the HIP path.
"""
import numpy as np


def dgemm(transa, transb, alpha, A, B, beta, C):
    """A, B, C: 2-D float64 arrays (row-major as given); returns the new C (M x N) as float64."""
    opA = np.asarray(A, dtype=np.float64).T if transa else np.asarray(A, dtype=np.float64)
    opB = np.asarray(B, dtype=np.float64).T if transb else np.asarray(B, dtype=np.float64)
    M, K = opA.shape
    K2, N = opB.shape
    if K != K2 or np.shape(C) != (M, N):
        raise ValueError("shapes do not agree")
    out = np.zeros((M, N), dtype=np.longdouble)
    if alpha != 0:
        a = opA.astype(np.longdouble)
        b = opB.astype(np.longdouble)
        for k in range(K):                         # k ascending, one rank-1 update per k
            out += np.multiply.outer(a[:, k], b[k, :])
        out *= np.longdouble(alpha)
    if beta != 0:
        out += np.longdouble(beta) * np.asarray(C, dtype=np.float64).astype(np.longdouble)
    return out.astype(np.float64)
