"""Pins of the generic bilinear oracle (Section 6.6: any <n0,n0,n0;q> scheme under the same recursion), no GPU."""
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


@pytest.mark.parametrize("scheme", [0, 1, 2, 3])
def test_tables_satisfy_the_bilinear_identity(bil, scheme):
    # sum_i U[i][a] V[i][b] W[c][i] must be 1 exactly when (a, b, c) is a term of the n0 x n0 product, else 0:
    # the defining (Brent) equations of a matrix multiplication scheme, independent of any implementation
    U, V, W, n0 = bil.tables(scheme)
    assert (n0, U.shape[0]) == {0: (2, 7), 1: (2, 8), 2: (3, 23), 3: (3, 27)}[scheme]
    assert set(np.unique(np.concatenate([U.ravel(), V.ravel(), W.ravel()]))) <= {-1, 0, 1}
    blocks = [(r, c) for r in range(n0) for c in range(n0)]
    for a, (ar, ac) in enumerate(blocks):
        for b, (br, bc) in enumerate(blocks):
            for c, (cr, cc) in enumerate(blocks):
                want = 1 if (ac == br and ar == cr and bc == cc) else 0
                assert int(np.sum(U[:, a] * V[:, b] * W[c, :])) == want, (a, b, c)


def test_laderman_is_a_fast_scheme(bil):
    # Section 6.6.2: q < n0^3 products and exponent w0 = log_n0 q; 23 < 27 and log_3 23 = 2.854 < 3.
    U, V, W, n0 = bil.tables(bil.LADERMAN)
    q = U.shape[0]
    assert q == 23 < n0 ** 3 and math.log(q, n0) == pytest.approx(2.854, abs=1e-3)
    assert [int(np.count_nonzero(W[c])) for c in range(9)] == [3, 7, 7, 7, 5, 5, 7, 5, 5]
    assert sorted(int(np.count_nonzero(U[i])) for i in range(q)) == sorted(int(np.count_nonzero(V[i])) for i in range(q))
    # seven of the products are plain block products (m6, m14, m19 .. m23)
    assert sum(1 for i in range(q) if np.count_nonzero(U[i]) == 1 and np.count_nonzero(V[i]) == 1) == 7


@pytest.mark.parametrize("scheme", [0, 1])
@pytest.mark.parametrize("n,levels", [(2, 1), (8, 2), (24, 3), (96, 4), (100, 2)])
def test_integer_products_exact(bil, scheme, n, levels):
    A = inputs.matrix(n, 11 + n, 0, "integer")
    B = inputs.matrix(n, 11 + n, 1, "integer")
    ref = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(bil.gemm(A, B, levels, scheme), ref)


@pytest.mark.parametrize("scheme", [2, 3])
@pytest.mark.parametrize("n,levels", [(3, 1), (9, 2), (27, 3), (54, 2), (81, 4), (90, 2)])
def test_integer_products_exact_on_three_by_three_blocks(bil, scheme, n, levels):
    A = inputs.matrix(n, 31 + n, 0, "integer")
    B = inputs.matrix(n, 31 + n, 1, "integer")
    ref = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(bil.gemm(A, B, levels, scheme), ref)
    if n == 9:
        brute = [[sum(int(A[i, k]) * int(B[k, j]) for k in range(n)) for j in range(n)] for i in range(n)]
        assert bil.gemm(A, B, levels, scheme).tolist() == [[float(v) for v in row] for row in brute]


def test_block_products_do_not_commute(bil):
    """A scheme that is only right for commuting entries (a b = b a) fails on matrix blocks: asymmetric operands
    through one Laderman step on 2 x 2 blocks (n = 6) and through steps of different schemes."""
    n = 6
    A = np.arange(1.0, n * n + 1).reshape(n, n)
    B = np.triu(np.ones((n, n))) * np.arange(1.0, n + 1)[None, :] - np.tril(np.ones((n, n)), -2)
    ref = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert not np.array_equal(ref, B @ A)
    assert np.array_equal(bil.gemm(A, B, 1, bil.LADERMAN), ref)
    assert np.array_equal(bil.gemm(A, B, 2, [bil.LADERMAN, bil.STRASSEN]), ref)
    assert np.array_equal(bil.gemm(A, B, 2, [bil.STRASSEN, bil.LADERMAN]), ref)


@pytest.mark.parametrize("schemes", [[0, 2], [2, 0], [2, 1, 0], [0, 2, 2], [3, 0], [2, 3], [0, 0, 2, 1]])
def test_mixed_levels_exact(bil, schemes):
    radix = 1
    for s in schemes:
        radix *= bil.tables(s)[3]
    n = radix * 5
    A = inputs.matrix(n, 3 + n, 0, "integer")
    B = inputs.matrix(n, 3 + n, 1, "integer")
    ref = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(bil.gemm(A, B, len(schemes), schemes), ref)
    with pytest.raises(RuntimeError):
        bil.gemm(A[: n - 1, : n - 1], B[: n - 1, : n - 1], len(schemes), schemes)      # not a multiple of the radix product


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


def test_operation_counts_on_three_by_three_blocks(bil):
    # F(n) = q F(n / n0) + a (n / n0)^2 with F(m) = 2 m^3 - m^2 at the leaves, a = the block additions of one
    # step counted from the tables (terms - 1 per combination); in closed form
    # F(n) = q^L (2 m^3 - m^2) + a sum_i q^i (n / 3^(i+1))^2
    n, levels = 54, 2
    m = n // 3 ** levels
    A = inputs.matrix(n, 1, 0, "integer")
    B = inputs.matrix(n, 1, 1, "integer")
    for scheme, q in ((bil.LADERMAN, 23), (bil.CLASSICAL27, 27)):
        U, V, W, n0 = bil.tables(scheme)
        a = int(sum(np.count_nonzero(r) - 1 for r in U) + sum(np.count_nonzero(r) - 1 for r in V) + sum(np.count_nonzero(r) - 1 for r in W))
        bil.reset_counters(); bil.gemm(A, B, levels, scheme); c = bil.counters()
        assert c["leaf_calls"] == q ** levels
        assert c["block_add"] == a * sum(q ** i * (n // 3 ** (i + 1)) ** 2 for i in range(levels))
        total = c["leaf_mul"] + c["leaf_add"] + c["block_add"]
        assert total == q ** levels * (2 * m ** 3 - m * m) + a * sum(q ** i * (n // 3 ** (i + 1)) ** 2 for i in range(levels))
        if scheme == bil.CLASSICAL27:
            assert a == 18 and total == 2 * n ** 3 - n * n          # exactly the classical algorithm's operations
        else:
            assert total < 2 * n ** 3 - n * n or levels < 3         # fewer products; additions weigh at this small n
    # the product count alone: 23^L against 27^L leaf products
    assert 23 ** 2 < 27 ** 2


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
    # three-by-three blocks
    n, levels = 162, 3
    A = inputs.matrix(n, 4, 0, "uniform")
    B = inputs.matrix(n, 4, 1, "uniform")
    ref = (A.astype(np.longdouble) @ B.astype(np.longdouble)).astype(np.float64)
    for scheme in (2, 3, [2, 0, 2]):
        lv = 3
        nn = n if not isinstance(scheme, list) else n
        got = bil.gemm(A, B, lv, scheme) if not isinstance(scheme, list) else bil.gemm(A[:108, :108], B[:108, :108], lv, scheme)
        want = ref if not isinstance(scheme, list) else (A[:108, :108].astype(np.longdouble) @ B[:108, :108].astype(np.longdouble)).astype(np.float64)
        assert np.max(np.abs(got - want)) <= 1e-10 * nn
    comp = n * np.finfo(float).eps * (np.abs(A) @ np.abs(B))
    assert np.all(np.abs(bil.gemm(A, B, levels, 3) - ref) <= comp)
