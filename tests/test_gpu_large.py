"""The three large configurations at full size, in the launch configuration the benchmark times.

The CPU oracle cannot finish these in seconds, so they are checked on what it CAN compute one by one and on
properties that hold at any size:
  * sampled entries C_ij against the oracle's definition-level dot product (long double accumulation) of
    row i of A and column j of B, both regenerated on the host from the counter-based generator;
  * Freivalds: C x against A (B x) for 8 random +-1 vectors, using torch's own GEMM (not this library);
  * integer-valued inputs, for which every intermediate is an exact integer: sampled entries and the
    Freivalds vectors must then agree EXACTLY.
Tolerance: 1e-10 * n * max|A| * max|B| per entry (the build's stated bar).
"""
import gc

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _free():
    gc.collect()
    torch.cuda.empty_cache()


def _sample_indices(n, count, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, n, size=(count, 2))
    idx[0] = (0, 0)
    idx[1] = (n - 1, n - 1)
    idx[2] = (n // 2 - 1, n // 2)        # straddles the top-level quadrant seam
    return idx


def _check_product(oracle, cfg, dist, schedule, host_pair=None, samples=24):
    n, levels, seed = cfg["n"], cfg["levels"], cfg["seed"]
    if host_pair is None:
        A = torch.empty((n, n), dtype=torch.float64, device=DEV)
        B = torch.empty((n, n), dtype=torch.float64, device=DEV)
        inputs.fill_device(A, n, seed, 0, dist)
        inputs.fill_device(B, n, seed, 1, dist)
    else:
        A = torch.from_numpy(host_pair[0]).to(DEV)
        B = torch.from_numpy(host_pair[1]).to(DEV)
    C = torch.empty((n, n), dtype=torch.float64, device=DEV)
    free, _ = torch.cuda.mem_get_info()
    if schedule is None:
        schedule = sw.sw_plan_schedule(n, levels, int(free - (2 << 30)))
    need = sw.sw_plan_workspace(n, levels, schedule, int(free - (2 << 30)))   # as bench.py does
    assert sw.sw_plan_memory(n, levels, schedule) <= need <= free, f"schedule {schedule} needs {need} bytes, {free} free"
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    sw.sw_gemm_ex(n, A, n, B, n, C, n, levels, schedule, ws)
    torch.cuda.synchronize()
    del ws
    _free()

    absmax = lambda t: max(float(t[r:r + 4096].abs().max()) for r in range(0, n, 4096))   # no n x n temporary
    amax, bmax = absmax(A), absmax(B)
    tol = 1e-10 * n * amax * bmax
    exact = dist == "integer"

    # sampled entries against the definition
    idx = _sample_indices(n, samples, seed)
    all_cols = np.arange(n)
    worst = 0.0
    for i, j in idx:
        if host_pair is None:
            a_row = inputs.block(n, seed, 0, dist, [i], all_cols).ravel()
            b_col = inputs.block(n, seed, 1, dist, all_cols, [j]).ravel()
        else:
            a_row, b_col = host_pair[0][i], np.ascontiguousarray(host_pair[1][:, j])
        ref = oracle.entry(a_row, b_col)
        got = float(C[i, j])
        if exact:
            assert got == ref, (i, j, got, ref)
        worst = max(worst, abs(got - ref))
    assert worst <= tol, (worst, tol)

    # Freivalds with 8 vectors of +-1 (their 1-norm is n)
    g = torch.Generator(device="cpu").manual_seed(seed)
    X = (torch.randint(0, 2, (n, 8), generator=g, dtype=torch.int64) * 2 - 1).to(torch.float64).to(DEV)
    y1 = C @ X
    y2 = A @ (B @ X)
    diff = float((y1 - y2).abs().max())
    if exact:
        assert diff == 0.0
    assert diff <= tol, (diff, tol)
    # a corrupted entry of that size would be seen: the check has teeth at the tolerance
    noise = diff
    assert noise < 0.5 * tol or exact
    del A, B, C, X, y1, y2
    _free()
    return schedule, worst, diff


def test_configuration_3(oracle):
    cfg = inputs.CONFIGS[2]
    pair = inputs.pair(cfg)                      # standard normal: generated on the host and uploaded
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], cfg["schedule"], host_pair=pair)
    print(f"cfg3 {s}: sampled max err {worst:.3e}, Freivalds {diff:.3e}")


def test_configuration_3_integer(oracle):
    cfg = inputs.CONFIGS[2]
    _check_product(oracle, cfg, "integer", cfg["schedule"])


def test_configuration_4(oracle):
    cfg = inputs.CONFIGS[3]
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], cfg["schedule"])
    print(f"cfg4 {s}: sampled max err {worst:.3e}, Freivalds {diff:.3e}")
    _check_product(oracle, cfg, "integer", None)          # the planner's own order, exact arithmetic


def test_configuration_5(oracle):
    cfg = inputs.CONFIGS[4]
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], None)
    print(f"cfg5 {s}: sampled max err {worst:.3e}, Freivalds {diff:.3e}")
    assert s == "DDDBB"


def test_peeled_size_near_configuration_5(oracle):
    # n = 94080 + 17: three more padded matrices would not fit in HBM; peeling needs no copies
    cfg = dict(inputs.CONFIGS[4], n=94097)
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL)
    try:
        s, worst, diff = _check_product(oracle, cfg, "integer", None)
        assert s == "DDDBB"
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


def test_configuration_5_integer(oracle):
    cfg = inputs.CONFIGS[4]
    _check_product(oracle, cfg, "integer", None)


def test_large_rectangular_product_freivalds():
    """30000 x 20000 x 25000 through four rectangular steps in the planner's order, integer-valued operands:
    C x must equal A (B x) exactly for 8 random +-1 vectors (every value involved is an exact integer)."""
    M, N, K, levels = 30000, 20000, 25000, 4
    A = torch.empty((M, K), dtype=torch.float64, device=DEV)
    B = torch.empty((K, N), dtype=torch.float64, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(5)
    A.copy_(torch.randint(-8, 9, (M, K), generator=g, device=DEV, dtype=torch.int32))
    B.copy_(torch.randint(-8, 9, (K, N), generator=g, device=DEV, dtype=torch.int32))
    C = torch.full((M, N), float("nan"), dtype=torch.float64, device=DEV)
    free, _ = torch.cuda.mem_get_info()
    ws = torch.empty(int(min(free - (2 << 30), 40 << 30)), dtype=torch.uint8, device=DEV)
    sw.sw_gemm_rect(M, N, K, A, K, B, N, C, N, levels, None, ws)
    torch.cuda.synchronize()
    gc_ = torch.Generator(device="cpu").manual_seed(9)
    for _ in range(8):
        x = (torch.randint(0, 2, (N,), generator=gc_, dtype=torch.int64) * 2 - 1).to(torch.float64).to(DEV)
        assert torch.equal(torch.mv(C, x), torch.mv(A, torch.mv(B, x)))
    del ws, A, B, C
    _free()
