"""Pins of the general-product oracle (alpha, beta, transposes, rectangular shapes), no GPU."""
import os
import sys

import numpy as np
import pytest

from paper_1202_3173_amd import inputs

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle"))
import sw_dgemm  # noqa: E402


def rect(rows, cols, seed, which, dist="integer"):
    n = max(rows, cols)
    return np.ascontiguousarray(inputs.matrix(n, seed, which, dist)[:rows, :cols])


def test_hand_worked_case():
    # 2 x 3 times 3 x 2, worked by hand: [[1,2,3],[4,5,6]] * [[1,0],[0,1],[2,2]] = [[7,8],[16,17]]
    A = np.array([[1.0, 2, 3], [4, 5, 6]])
    B = np.array([[1.0, 0], [0, 1], [2, 2]])
    C = np.array([[1.0, 1], [1, 1]])
    assert np.array_equal(sw_dgemm.dgemm(False, False, 2.0, A, B, -1.0, C), [[13, 15], [31, 33]])
    # the same through both transposes: op(A) = (A^T)^T, op(B) = (B^T)^T
    assert np.array_equal(sw_dgemm.dgemm(True, True, 2.0, A.T.copy(), B.T.copy(), -1.0, C), [[13, 15], [31, 33]])
    # a swapped operand order or a missing transpose gives another shape or another value
    assert not np.array_equal(sw_dgemm.dgemm(True, False, 1.0, A[:, :2], A[:, :2], 0.0, np.zeros((2, 2))),
                              sw_dgemm.dgemm(False, False, 1.0, A[:, :2], A[:, :2], 0.0, np.zeros((2, 2))))


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_against_blas_and_exact_integers(ta, tb):
    from scipy.linalg.blas import dgemm as blas_dgemm
    M, N, K = 37, 53, 29
    A = rect(K, M, 1, 0) if ta else rect(M, K, 1, 0)
    B = rect(N, K, 1, 1) if tb else rect(K, N, 1, 1)
    C = rect(M, N, 2, 0)
    for alpha, beta in [(1.0, 0.0), (2.0, -0.5), (0.0, 3.0), (-1.0, 1.0)]:
        got = sw_dgemm.dgemm(ta, tb, alpha, A, B, beta, C)
        opA = A.T if ta else A
        opB = B.T if tb else B
        exact = alpha * (opA.astype(np.int64) @ opB.astype(np.int64)) + beta * C      # small integers: exact in fp64
        assert np.array_equal(got, exact)
        ref = blas_dgemm(alpha, A, B, beta=beta, c=C, trans_a=ta, trans_b=tb)       # the library routine
        assert np.array_equal(got, ref)


def test_beta_zero_ignores_c_and_alpha_zero_ignores_operands():
    A = rect(5, 4, 3, 0)
    B = rect(4, 6, 3, 1)
    C = np.full((5, 6), np.nan)
    assert np.array_equal(sw_dgemm.dgemm(False, False, 1.0, A, B, 0.0, C), A @ B)
    An = np.full((5, 4), np.nan)
    C1 = rect(5, 6, 4, 0)
    assert np.array_equal(sw_dgemm.dgemm(False, False, 0.0, An, B, 2.0, C1), 2.0 * C1)


def test_real_inputs_close_to_library_product():
    M, N, K = 64, 40, 96
    A = rect(M, K, 5, 0, "uniform")
    B = rect(K, N, 5, 1, "rowscaled")
    C = rect(M, N, 6, 0, "uniform")
    got = sw_dgemm.dgemm(False, False, 1.5, A, B, 0.25, C)
    ref = 1.5 * (A @ B) + 0.25 * C
    assert np.max(np.abs(got - ref)) <= 4 * K * np.finfo(float).eps * np.max(np.abs(A)) * np.max(np.abs(B)) * 1.5
