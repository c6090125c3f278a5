"""Other block schemes (2 x 2 and 3 x 3 blocks) on the BFS/DFS machinery (Section 6.6) on the GPU against the bilinear oracle.

Bar as for the main path: within 1e-10 * n * max|A| * max|B| on real inputs (the leaf products sum in another
order than the oracle's), bit for bit on integer-valued inputs, and no dependence on the BFS/DFS order at all.
"""
import os
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle"))
pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ORACLE_SCHEME = {sw.SW_SCHEME_STRASSEN: 0, sw.SW_SCHEME_CLASSICAL: 1, sw.SW_SCHEME_LADERMAN: 2, sw.SW_SCHEME_CLASSICAL3: 3}


@pytest.fixture(scope="module")
def bil(oracle):
    import sw_bilinear
    sw_bilinear.lib()
    return sw_bilinear


def run(A, B, levels, schedule, scheme, slack=0):
    n = A.shape[0]
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
    need = sw.sw_plan_memory_bilinear(n, levels, schedule, scheme)
    ws = torch.empty(max(need + slack, 256), dtype=torch.uint8, device=DEV)
    sw.sw_set_workspace(ws)
    sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
    try:
        sw.sw_gemm_bilinear(n, dA, dB, C, levels, schedule, scheme)
        torch.cuda.synchronize()
    finally:
        sw.sw_set_workspace(None)
        sw.sw_set_stream(0)
    assert torch.equal(dA.cpu(), torch.from_numpy(A)) and torch.equal(dB.cpu(), torch.from_numpy(B)), "inputs changed"
    return C.cpu().numpy()


CASES = [(2, 1, "B"), (2, 1, "D"), (64, 2, "BD"), (96, 3, "DBD"), (264, 2, "DD"), (520, 3, "BBB"), (1000, 2, "DB"),
         (333, 2, "BD"), (777, 3, "DDB"), (1536, 4, "DBDB")]


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_CLASSICAL])
@pytest.mark.parametrize("n,levels,schedule", CASES)
def test_integer_products_bit_exact(bil, scheme, n, levels, schedule):
    A = inputs.matrix(n, 70 + n, 0, "integer")
    B = inputs.matrix(n, 70 + n, 1, "integer")
    got = run(A, B, levels, schedule, scheme)
    exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(got, exact)
    if n % (1 << levels) == 0 and n <= 520:
        assert np.array_equal(got, bil.gemm(A, B, levels, ORACLE_SCHEME[scheme]))


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_CLASSICAL])
@pytest.mark.parametrize("n,levels,schedule", [(64, 2, "BD"), (520, 3, "BBB"), (520, 3, "DDD"), (1024, 3, "DBD"), (1000, 2, "DB")])
def test_real_products_within_tolerance(bil, scheme, n, levels, schedule):
    A = inputs.matrix(n, 5 + n, 0, "uniform")
    B = inputs.matrix(n, 5 + n, 1, "rowscaled")
    got = run(A, B, levels, schedule, scheme)
    if n % (1 << levels) == 0:
        ref = bil.gemm(A, B, levels, ORACLE_SCHEME[scheme])
    else:   # the oracle takes multiples of 2^levels only: zero padding does not change the product
        npad = -(-n // (1 << levels)) * (1 << levels)
        Ap = np.zeros((npad, npad)); Ap[:n, :n] = A
        Bp = np.zeros((npad, npad)); Bp[:n, :n] = B
        ref = bil.gemm(Ap, Bp, levels, ORACLE_SCHEME[scheme])[:n, :n]
    bar = 1e-10 * n * float(np.max(np.abs(A))) * float(np.max(np.abs(B)))
    assert np.max(np.abs(got - ref)) <= bar
    if scheme == sw.SW_SCHEME_CLASSICAL:
        # the recursive classical algorithm keeps the component-wise bound of the classical one (Section 6.1)
        exact = (A.astype(np.longdouble) @ B.astype(np.longdouble)).astype(np.float64)
        assert np.all(np.abs(got - exact) <= n * np.finfo(float).eps * (np.abs(A) @ np.abs(B)))


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_CLASSICAL])
def test_every_step_order_gives_the_same_bits(scheme):
    n, levels = 448, 3
    A = inputs.matrix(n, 8, 0, "uniform")
    B = inputs.matrix(n, 8, 1, "uniform")
    first = None
    for mask in range(1 << levels):
        schedule = "".join("B" if (mask >> i) & 1 else "D" for i in range(levels))
        got = run(A, B, levels, schedule, scheme)
        if first is None:
            first = got
        assert np.array_equal(got, first), schedule


def test_planned_order_and_winograd_forwarding():
    n, levels = 512, 3
    A = inputs.matrix(n, 9, 0, "integer")
    B = inputs.matrix(n, 9, 1, "integer")
    exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    # schedule None: the library plans for the workspace it was given (here: room for all-BFS)
    slack = sw.sw_plan_memory_bilinear(n, levels, "BBB", sw.SW_SCHEME_STRASSEN)
    assert np.array_equal(run(A, B, levels, None, sw.SW_SCHEME_STRASSEN, slack=slack), exact)
    # scheme 0 is the Strassen-Winograd product itself
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.empty((n, n), dtype=torch.float64, device=DEV)
    ws = torch.empty(sw.sw_plan_memory(n, levels, "BDB"), dtype=torch.uint8, device=DEV)
    sw.sw_set_workspace(ws)
    try:
        sw.sw_gemm_bilinear(n, dA, dB, C, levels, "BDB", sw.SW_SCHEME_WINOGRAD)
        torch.cuda.synchronize()
    finally:
        sw.sw_set_workspace(None)
    assert np.array_equal(C.cpu().numpy(), exact)


def test_errors():
    n = 64
    A = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    C = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    with pytest.raises(sw.SwError) as e:
        sw.sw_gemm_bilinear(n, A, A, C, 1, "B", 7)
    assert e.value.code == -1
    sw.sw_set_workspace(None)
    with pytest.raises(sw.SwError) as e:
        sw.sw_gemm_bilinear(n, A, A, C, 1, "B", sw.SW_SCHEME_STRASSEN)
    assert e.value.code == -2


def test_seeded_sweep_is_exact():
    """Thirty seeded combinations of scheme, size (odd ones are padded), depth and step order on integers."""
    rng = np.random.default_rng(4242)
    for case in range(30):
        scheme = int(rng.choice([sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_CLASSICAL]))
        levels = int(rng.integers(0, 4))
        n = int(rng.integers(1 << levels, 500))
        schedule = "".join(rng.choice(["B", "D"]) for _ in range(levels))
        A = inputs.matrix(n, 900 + case, 0, "integer")
        B = inputs.matrix(n, 900 + case, 1, "integer")
        exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
        assert np.array_equal(run(A, B, levels, schedule, scheme), exact), (case, scheme, n, levels, schedule)


# ---- 3 x 3 blocks (Section 6.6.2) and mixed radices -------------------------------------------------------------------

def run_levels(A, B, schedule, schemes, slack=0):
    n = A.shape[0]
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
    need = sw.sw_plan_memory_bilinear_levels(n, schedule, schemes)
    ws = torch.empty(max(need + slack, 256), dtype=torch.uint8, device=DEV)
    sw.sw_set_workspace(ws)
    sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
    try:
        sw.sw_gemm_bilinear_levels(n, dA, dB, C, schedule, schemes)
        torch.cuda.synchronize()
    finally:
        sw.sw_set_workspace(None)
        sw.sw_set_stream(0)
    assert torch.equal(dA.cpu(), torch.from_numpy(A)) and torch.equal(dB.cpu(), torch.from_numpy(B)), "inputs changed"
    return C.cpu().numpy()


CASES3 = [(3, 1, "B"), (3, 1, "D"), (81, 2, "BD"), (81, 2, "DB"), (270, 3, "DBD"), (486, 3, "BBB"), (1000, 2, "DB"),
          (333, 2, "BD"), (700, 3, "DDB"), (1458, 4, "DBDD")]


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_CLASSICAL3])
@pytest.mark.parametrize("n,levels,schedule", CASES3)
def test_three_by_three_integer_products_bit_exact(bil, scheme, n, levels, schedule):
    A = inputs.matrix(n, 170 + n, 0, "integer")
    B = inputs.matrix(n, 170 + n, 1, "integer")
    got = run(A, B, levels, schedule, scheme)
    exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert np.array_equal(got, exact)
    if n % (3 ** levels) == 0 and n <= 486:
        assert np.array_equal(got, bil.gemm(A, B, levels, ORACLE_SCHEME[scheme]))


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_CLASSICAL3])
@pytest.mark.parametrize("n,levels,schedule", [(81, 2, "BD"), (486, 3, "BBB"), (486, 3, "DDD"), (972, 3, "DBD"), (1000, 2, "DB")])
def test_three_by_three_real_products_within_tolerance(bil, scheme, n, levels, schedule):
    A = inputs.matrix(n, 5 + n, 0, "uniform")
    B = inputs.matrix(n, 5 + n, 1, "rowscaled")
    got = run(A, B, levels, schedule, scheme)
    r = 3 ** levels
    npad = -(-n // r) * r          # the oracle takes multiples of 3^levels only: zero padding does not change the product
    Ap = np.zeros((npad, npad)); Ap[:n, :n] = A
    Bp = np.zeros((npad, npad)); Bp[:n, :n] = B
    ref = bil.gemm(Ap, Bp, levels, ORACLE_SCHEME[scheme])[:n, :n]
    bar = 1e-10 * n * float(np.max(np.abs(A))) * float(np.max(np.abs(B)))
    assert np.max(np.abs(got - ref)) <= bar
    if scheme == sw.SW_SCHEME_CLASSICAL3:
        exact = (A.astype(np.longdouble) @ B.astype(np.longdouble)).astype(np.float64)
        assert np.all(np.abs(got - exact) <= n * np.finfo(float).eps * (np.abs(A) @ np.abs(B)))


@pytest.mark.parametrize("scheme", [sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_CLASSICAL3])
def test_three_by_three_every_step_order_gives_the_same_bits(bil, scheme):
    n, levels = 486, 3
    A = inputs.matrix(n, 8, 0, "uniform")
    B = inputs.matrix(n, 8, 1, "uniform")
    first = None
    for mask in range(1 << levels):
        schedule = "".join("B" if (mask >> i) & 1 else "D" for i in range(levels))
        got = run(A, B, levels, schedule, scheme)
        if first is None:
            first = got
        assert np.array_equal(got, first), schedule
    # ... and on integers every order is the exact product
    Ai = inputs.matrix(n, 12, 0, "integer")
    Bi = inputs.matrix(n, 12, 1, "integer")
    exact = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64)
    for schedule in ("DDD", "BDB", "BBB"):
        assert np.array_equal(run(Ai, Bi, levels, schedule, scheme), exact)


MIXED = [([sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_LADERMAN], "BD"), ([sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_STRASSEN], "DB"),
         ([sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_CLASSICAL, sw.SW_SCHEME_STRASSEN], "BDB"),
         ([sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_LADERMAN], "DBB"),
         ([sw.SW_SCHEME_CLASSICAL3, sw.SW_SCHEME_LADERMAN], "BB"),
         ([sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_CLASSICAL3], "DBDB")]


@pytest.mark.parametrize("schemes,schedule", MIXED)
def test_mixed_radices(bil, schemes, schedule):
    """Steps on 2 x 2 and 3 x 3 blocks in one recursion: exact on integers (also at a size the radix product does
    not divide), the oracle's bits on integers, and inside the tolerance on real inputs."""
    radix = int(np.prod([sw.SCHEME_BASE[s] for s in schemes]))
    oracle_schemes = [ORACLE_SCHEME[s] for s in schemes]
    for n in (radix * 7, radix * 7 + 5):
        A = inputs.matrix(n, 300 + n, 0, "integer")
        B = inputs.matrix(n, 300 + n, 1, "integer")
        got = run_levels(A, B, schedule, schemes)
        assert np.array_equal(got, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64))
        if n % radix == 0:
            assert np.array_equal(got, bil.gemm(A, B, len(schemes), oracle_schemes))
    n = radix * 11
    A = inputs.matrix(n, 5, 0, "uniform")
    B = inputs.matrix(n, 5, 1, "uniform")
    got = run_levels(A, B, schedule, schemes)
    ref = bil.gemm(A, B, len(schemes), oracle_schemes)
    assert np.max(np.abs(got - ref)) <= 1e-10 * n
    # the other extreme of the step orders gives the same bits
    other = "".join("D" if ch == "B" else "B" for ch in schedule)
    assert np.array_equal(run_levels(A, B, other, schemes), got)


def test_levels_errors_and_planned_order():
    n = 90
    A = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    C = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    with pytest.raises(sw.SwError) as e:
        sw.sw_gemm_bilinear_levels(n, A, A, C, "BB", [sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_WINOGRAD])
    assert e.value.code == sw.SW_EINVAL
    with pytest.raises(sw.SwError) as e:                     # 3^5 = 243 parts of 90 rows
        sw.sw_gemm_bilinear_levels(n, A, A, C, "DDDDD", [sw.SW_SCHEME_LADERMAN] * 5)
    assert e.value.code == sw.SW_EINVAL
    # schedule None: the library plans for the workspace it has
    n = 324
    Ah = inputs.matrix(n, 3, 0, "integer")
    Bh = inputs.matrix(n, 3, 1, "integer")
    schemes = [sw.SW_SCHEME_LADERMAN, sw.SW_SCHEME_STRASSEN]
    slack = sw.sw_plan_memory_bilinear_levels(n, "BB", schemes)
    got = run_levels(Ah, Bh, None, schemes, slack=slack)
    assert np.array_equal(got, (Ah.astype(np.int64) @ Bh.astype(np.int64)).astype(np.float64))
