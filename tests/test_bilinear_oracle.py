"""Pins of the generic bilinear oracle (Section 6.6: any <2,2,2;q> scheme under the same recursion), no GPU."""
import math
import os
import sys

import numpy as np
import pytest

from paper_1202_3173_amd import inputs

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle"))


@pytest.fixture(scope="module")
def bil(oracle):
    import sw_bilinear
    sw_bilinear.lib()
    return sw_bilinear


@pytest.mark.parametrize("scheme", [0, 1])
def test_tables_satisfy_the_bilinear_identity(bil, scheme):
    # sum_i U[i][a] V[i][b] W[c][i] must be 1 exactly when (a, b, c) is a term of the 2 x 2 product, else 0:
    # the defining (Brent) equations of a matrix multiplication scheme, independent of any implementation
    U, V, W = bil.tables(scheme)
    quad = [(0, 0), (0, 1), (1, 0), (1, 1)]
    for a, (ar, ac) in enumerate(quad):
        for b, (br, bc) in enumerate(quad):
            for c, (cr, cc) in enumerate(quad):
                want = 1 if (ac == br and ar == cr and bc == cc) else 0
                assert int(np.sum(U[:, a] * V[:, b] * W[c, :])) == want, (a, b, c)


@pytest.mark.parametrize("scheme", [0, 1])
@pytest.mark.parametrize("n,levels", [(2, 1), (8, 2), (24, 3), (96, 4), (100, 2)])
def test_integer_products_exact(bil, scheme, n, levels):
    A = inputs.matrix(n, 11 + n, 0, "integer")
    B = inputs.matrix(n, 11 + n, 1, "integer")
    ref = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(bil.gemm(A, B, levels, scheme), ref)


def test_operation_counts(bil):
    n, levels = 64, 3
    n0 = n >> levels
    A = inputs.matrix(n, 1, 0, "integer")
    B = inputs.matrix(n, 1, 1, "integer")
    # Strassen: 7 products and 18 additions per step (Section 2.2; the recurrences of Section 3.3.2):
    # F(n) = c n^w0 - 6 n^2 with F(n0) = 2 n0^3 - n0^2
    bil.reset_counters(); bil.gemm(A, B, levels, bil.STRASSEN); c = bil.counters()
    assert c["leaf_calls"] == 7 ** levels
    assert c["block_add"] == 18 * sum(7 ** i * (n >> (i + 1)) ** 2 for i in range(levels))
    total = c["leaf_mul"] + c["leaf_add"] + c["block_add"]
    w0 = math.log2(7)
    cs = (2 * n0 + 5) / n0 ** (w0 - 2)
    assert total == pytest.approx(cs * n ** w0 - 6 * n * n, rel=1e-12)
    assert total == (2 * n0 + 5) * n0 * n0 * 7 ** levels - 6 * n * n
    # recursive classical: exactly the 2 n^3 - n^2 operations of the classical algorithm
    bil.reset_counters(); bil.gemm(A, B, levels, bil.CLASSICAL8); c = bil.counters()
    assert c["leaf_calls"] == 8 ** levels
    assert c["leaf_mul"] + c["leaf_add"] + c["block_add"] == 2 * n ** 3 - n * n


def test_float_close_to_winograd_oracle_and_reference(bil, oracle):
    n, levels = 128, 3
    A = inputs.matrix(n, 4, 0, "uniform")
    B = inputs.matrix(n, 4, 1, "uniform")
    ref = (A.astype(np.longdouble) @ B.astype(np.longdouble)).astype(np.float64)
    for scheme in (0, 1):
        assert np.max(np.abs(bil.gemm(A, B, levels, scheme) - ref)) <= 1e-10 * n
    # the recursive classical scheme obeys the component-wise bound of the classical algorithm (Section 6.1)
    comp = n * np.finfo(float).eps * (np.abs(A) @ np.abs(B))
    assert np.all(np.abs(bil.gemm(A, B, levels, 1) - ref) <= comp)
