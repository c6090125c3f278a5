"""sw_dgemm (alpha, beta, transposes, rectangular shapes, automatic depth) on the GPU against the general-product
oracle.  Integer-valued operands with alpha, beta in {small integers, 1/2}: every intermediate is exact, so the
result must equal the oracle bit for bit; real operands: within 1e-10 * K * |alpha| * max|A| * max|B|."""
import os
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle"))
import sw_dgemm as oracle_dgemm  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rect(rows, cols, seed, which, dist):
    n = max(rows, cols)
    return np.ascontiguousarray(inputs.matrix(n, seed, which, dist)[:rows, :cols])


def stored(rows, cols, pad, seed, which, dist):
    """Host matrix and a device buffer that holds it with leading dimension cols + pad (padding NaN)."""
    H = rect(rows, cols, seed, which, dist)
    D = torch.full((rows, cols + pad), float("nan"), dtype=torch.float64, device=DEV)
    D[:, :cols] = torch.from_numpy(H).to(DEV)
    return H, D


def run(ta, tb, M, N, K, alpha, beta, levels, schedule, dist="integer", pads=(0, 0, 0), seed=1, extra_ws=0, c_nan=False,
        exact_reference=False):
    A, dA = stored(K if ta else M, M if ta else K, pads[0], seed, 0, dist)
    B, dB = stored(N if tb else K, K if tb else N, pads[1], seed, 1, dist)
    C, dC = stored(M, N, pads[2], seed + 1, 0, dist)
    if c_nan:
        dC[:, :N] = float("nan")
    if levels >= 0:
        need = sw.sw_plan_memory_dgemm(ta, tb, M, N, K, levels, schedule)
    else:
        need = 0
    ws = torch.empty(max(need + extra_ws, 256), dtype=torch.uint8, device=DEV)
    sw.sw_set_workspace(ws)
    sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
    try:
        sw.sw_dgemm(ta, tb, M, N, K, alpha, dA, dA.shape[1], dB, dB.shape[1], beta, dC, dC.shape[1], levels, schedule)
        torch.cuda.synchronize()
    finally:
        sw.sw_set_workspace(None)
        sw.sw_set_stream(0)
    got = dC.cpu().numpy()
    if pads[2]:
        assert np.all(np.isnan(got[:, N:])), "wrote into the padding of C"
    assert np.array_equal(dA.cpu().numpy()[:, :A.shape[1]], A) and np.array_equal(dB.cpu().numpy()[:, :B.shape[1]], B)
    if exact_reference:
        # too large for the entry-by-entry oracle; on small-integer operands every partial sum is an integer
        # below 2^53, so the fp64 library product is the exact product whatever its summation order
        ref = alpha * ((A.T if ta else A) @ (B.T if tb else B)) + beta * C
    else:
        ref = oracle_dgemm.dgemm(ta, tb, alpha, A, B, beta, np.zeros((M, N)) if c_nan else C)
    return got[:, :N], ref, A, B


SHAPES = [(128, 128, 128, 2, "BB"), (300, 200, 260, 2, "DB"), (200, 300, 260, 2, "BD"), (513, 257, 1030, 3, "DBB"),
          (96, 700, 96, 1, "B"), (1000, 64, 900, 0, ""), (257, 255, 129, 4, "DBDB"), (640, 640, 1280, 3, "BBB")]


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("M,N,K,levels,schedule", SHAPES)
def test_integer_operands_bit_exact(ta, tb, M, N, K, levels, schedule):
    got, ref, _, _ = run(ta, tb, M, N, K, 2.0, -0.5, levels, schedule, pads=(3, 0, 5))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_real_operands_within_tolerance(ta, tb):
    M, N, K = 700, 520, 900
    got, ref, A, B = run(ta, tb, M, N, K, 1.5, 0.25, 2, "DB", dist="uniform", pads=(0, 2, 0), seed=7)
    assert np.max(np.abs(got - ref)) <= 1e-10 * K * 1.5 * np.max(np.abs(A)) * np.max(np.abs(B))


def test_beta_zero_does_not_read_c_and_alpha_zero_does_not_read_operands():
    got, ref, _, _ = run(False, True, 260, 200, 300, 1.0, 0.0, 2, "BD", c_nan=True)
    assert np.array_equal(got, ref)
    M, N = 100, 90
    C = rect(M, N, 3, 0, "integer")
    dC = torch.from_numpy(C).to(DEV)
    sw.sw_set_workspace(None)
    sw.sw_dgemm(False, False, M, N, 50, 0.0, None, 50, None, N, 3.0, dC, N, 0, "")     # A, B not even given
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), 3.0 * C)
    sw.sw_dgemm(False, False, M, N, 0, 1.0, None, 1, None, N, 0.0, dC, N, 0, "")        # K = 0, beta = 0: zeros
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.zeros((M, N)))


@pytest.mark.parametrize("ta,tb", [(False, False), (True, True)])
def test_unscaled_product_goes_straight_into_c(ta, tb):
    # alpha = 1, beta = 0, one block along K: no temporary, no fold; C (NaN before, padded pitch) is simply written
    got, ref, _, _ = run(ta, tb, 512, 768, 256, 1.0, 0.0, 2, "DB", pads=(1, 2, 3), c_nan=True)
    assert np.array_equal(got, ref)


def test_automatic_depth():
    # with room to spare the library picks the depth itself; whatever it picks, integers stay exact
    M, N, K = 8300, 8200, 8400
    got, ref, _, _ = run(False, False, M, N, K, 1.0, 1.0, -1, None, extra_ws=4 << 30, exact_reference=True)
    assert np.array_equal(got, ref)
    assert sw.sw_plan_levels(8200, 3 << 30) >= 1      # so the call above did recurse
    # the square product takes the same choice with levels < 0
    n = 8200
    A = rect(n, n, 5, 0, "integer")
    B = rect(n, n, 5, 1, "integer")
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
    ws = torch.empty(3 << 30, dtype=torch.uint8, device=DEV)
    sw.sw_gemm_ex(n, dA, n, dB, n, C, n, -1, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), A @ B)
    del ws
    # and so does the convenience call that allocates C and the workspace itself
    assert np.array_equal(sw.matmul(dA, dB).cpu().numpy(), A @ B)


def test_errors():
    t = torch.zeros((64, 64), dtype=torch.float64, device=DEV)
    sw.sw_set_workspace(None)
    for args, code in [((False, False, 64, 64, 64, 1.0, t, 63, t, 64, 0.0, torch.zeros_like(t), 64, 1, "B"), -1),   # lda < K
                       ((False, False, 64, 64, 64, 1.0, t, 64, t, 64, 0.0, t, 64, 1, "B"), -1),                      # C is A
                       ((False, False, 64, 64, 2, 1.0, t, 64, t, 64, 0.0, torch.zeros_like(t), 64, 2, "BB"), -1),    # 2^levels > K
                       ((False, False, 64, 64, 64, 1.0, t, 64, t, 64, 0.0, torch.zeros_like(t), 64, 1, "B"), -2)]:   # no workspace
        with pytest.raises(sw.SwError) as e:
            sw.sw_dgemm(*args)
        assert e.value.code == code


def test_seeded_sweep_of_general_products_is_exact():
    """Thirty seeded combinations of shapes, transposes, leading-dimension padding, depths and coefficients on
    integer-valued operands: alpha and beta are small multiples of 1/2, so every value is exact in fp64 and the
    result must equal alpha * op(A) op(B) + beta * C bit for bit."""
    rng = np.random.default_rng(77)
    for case in range(30):
        levels = int(rng.integers(0, 4))
        lo = 1 << levels
        M, N, K = (int(rng.integers(lo, 420)) for _ in range(3))
        ta, tb = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        alpha = float(rng.choice([1.0, -1.0, 2.0, 0.5, 3.0]))
        beta = float(rng.choice([0.0, 1.0, -0.5, 2.0]))
        pads = tuple(int(x) for x in rng.integers(0, 4, size=3))
        got, ref, _, _ = run(ta, tb, M, N, K, alpha, beta, levels, None, pads=pads, seed=500 + case, exact_reference=True,
                             extra_ws=int(rng.integers(0, 2)) * (64 << 20))
        assert np.array_equal(got, ref), (case, M, N, K, ta, tb, alpha, beta, levels, pads)
