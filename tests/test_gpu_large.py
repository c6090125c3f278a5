"""The three large configurations at full size, in the launch configuration the benchmark times.

The CPU oracle cannot finish these in seconds, so they are checked on what it CAN compute and on properties
that hold at any size:
  * configurations 3 and 4: about a hundred whole rows and a hundred whole columns of C, element by element,
    against the oracle's strips of the definition; the rows and columns straddle every quadrant seam of every
    level (the multiples of the leaf size, one below and at), the 128-wide tile edges inside several leaves,
    the last partial tile of a leaf and the matrix border -- the places where an indexing mistake shows;
  * sampled entries C_ij against the oracle's definition-level dot product (long double accumulation) of
    row i of A and column j of B, both regenerated on the host from the counter-based generator; the samples
    are not random: they sit on the same seams, tile edges and partial tiles, in pairs that cross them;
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


def _marks(n, levels, want=None, seed=0):
    """Row (or column) indices where mistakes show: one below and at every multiple of the leaf size (the quadrant
    seams of all levels), the edges of the product kernel's 128-wide tiles and the last, partial tile inside the
    first, a middle and the last leaf, and the border; filled up to `want` with seeded random ones."""
    m = n >> levels
    marks = {0, n - 1}
    for b in range(m, n, m):
        marks |= {b - 1, b}
    last_tile = (m - 1) // 128 * 128                       # first row of the last tile of a leaf (partial unless 128 | m)
    for leaf in (0, (n // m) // 2, n // m - 1):
        base = leaf * m
        for t in (1, 127, 128, 129, last_tile - 1, last_tile, last_tile + 1, m - 2):
            if 0 <= t < m:
                marks.add(base + t)
    marks = sorted(marks)
    if want is not None and len(marks) < want:
        rng = np.random.default_rng(seed)
        rest = np.setdiff1d(rng.integers(0, n, size=4 * want), marks)
        marks = sorted(set(marks) | set(rest[: want - len(marks)].tolist()))
    return np.array(marks, dtype=np.int64)


def _few_marks(n, levels):
    """A short list of the same kind for the largest configuration, where every row costs a pass over 70 GB: the
    border, the seams of the top two levels and of the first and last leaf, tile edges and the partial tile."""
    m = n >> levels
    last_tile = (m - 1) // 128 * 128
    marks = {0, 127, 128, last_tile - 1, last_tile, m - 1, m, n // 4 - 1, n // 4, n // 2 - 1, n // 2, 3 * n // 4 - 1, 3 * n // 4,
             n - m - 1, n - m, n - m + last_tile, n - 1}
    return np.array(sorted(marks), dtype=np.int64)


def _sample_indices(n, levels, count):
    """Entries that cross the marks: every marked row with a marked column, walking both lists at coprime strides."""
    marks = _marks(n, levels)
    k = len(marks)
    idx = [(0, 0), (n - 1, n - 1), (n // 2 - 1, n // 2), (n // 2, n // 2 - 1)]
    import math
    stride = next(q for q in (7, 5, 11, 13, 17) if math.gcd(q, k) == 1)
    t = 0
    while len(idx) < count:
        idx.append((int(marks[t % k]), int(marks[(stride * t + 3) % k])))
        t += 1
    return np.array(idx[:count], dtype=np.int64)


def _check_strips(oracle, C, A_host, B_host, levels, tol, exact, want):
    """Whole rows and whole columns of the device result against the oracle's strips of the definition."""
    from concurrent.futures import ThreadPoolExecutor
    n = A_host.shape[0]
    if want == "few":
        rows = cols = _few_marks(n, levels)
    else:
        rows = _marks(n, levels, want, seed=1)
        cols = _marks(n, levels, want, seed=2)
    got_rows = C[torch.from_numpy(rows).to(C.device)].cpu().numpy()
    got_cols = C[:, torch.from_numpy(cols).to(C.device)].cpu().numpy()
    # the oracle is single-threaded; independent groups of rows / columns are handed to it from several threads
    per = 8 if len(rows) >= 48 else 2
    groups = lambda idx: [idx[k:k + per] for k in range(0, len(idx), per)]
    with ThreadPoolExecutor(12) as pool:
        ref_rows = np.concatenate(list(pool.map(lambda g: oracle.row_strip(A_host[g], B_host), groups(rows))), axis=0)
        ref_cols = np.concatenate(list(pool.map(lambda g: oracle.col_strip(A_host, np.ascontiguousarray(B_host[:, g])), groups(cols))), axis=1)
    if exact:
        assert np.array_equal(got_rows, ref_rows) and np.array_equal(got_cols, ref_cols)
    worst = max(float(np.max(np.abs(got_rows - ref_rows))), float(np.max(np.abs(got_cols - ref_cols))))
    assert worst <= tol, (worst, tol)
    return worst, len(rows), len(cols)


def _check_product(oracle, cfg, dist, schedule, host_pair=None, samples=64, strips=0):
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
    idx = _sample_indices(n, levels, samples)
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

    # whole rows and columns, element by element
    if strips:
        if host_pair is None:
            # the operands come from the seeded generator's device fill; tie the downloaded copies to the host generator
            Ah, Bh = A.cpu().numpy(), B.cpu().numpy()
            probe = np.array([0, n // 3, n - 1])
            assert np.array_equal(Ah[probe], inputs.block(n, seed, 0, dist, probe, all_cols))
            assert np.array_equal(Bh[:, probe], inputs.block(n, seed, 1, dist, all_cols, probe))
        else:
            Ah, Bh = host_pair
        w, nr, nc = _check_strips(oracle, C, Ah, Bh, levels, tol, exact, strips)
        print(f"{cfg['name']} {dist}: {nr} rows and {nc} columns element by element, max err {w:.3e} (tol {tol:.3e})")
        worst = max(worst, w)
        del Ah, Bh

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
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], cfg["schedule"], host_pair=pair, strips=128)
    print(f"cfg3 {s}: max err {worst:.3e}, Freivalds {diff:.3e}")


def test_configuration_3_integer(oracle):
    cfg = inputs.CONFIGS[2]
    _check_product(oracle, cfg, "integer", cfg["schedule"], strips=48)


def test_configuration_4(oracle):
    cfg = inputs.CONFIGS[3]
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], cfg["schedule"], strips=112)
    print(f"cfg4 {s}: max err {worst:.3e}, Freivalds {diff:.3e}")


def test_configuration_4_integer_planner_order(oracle):
    cfg = inputs.CONFIGS[3]
    _check_product(oracle, cfg, "integer", None, strips=80)          # the planner's own order, exact arithmetic


def test_configuration_5(oracle):
    cfg = inputs.CONFIGS[4]
    s, worst, diff = _check_product(oracle, cfg, cfg["dist"], None, samples=96, strips="few")
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


def test_peeled_at_every_level_near_configuration_5(oracle):
    # the same size with peeling level by level: 94097 and 5881 are the odd levels (94097 -> 47048 -> 23524 -> 11762 -> 5881 -> 2940)
    cfg = dict(inputs.CONFIGS[4], n=94097)
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL_LEVELS)
    try:
        s, worst, diff = _check_product(oracle, cfg, "integer", None)
        assert s == "DDDBB"
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


def test_configuration_5_integer(oracle):
    """The largest configuration on integer-valued inputs: sampled entries and Freivalds vectors exact, and 17 whole rows
    and 17 whole columns (border, top seams, leaf seams, tile edges) EQUAL to the oracle's strips of the definition."""
    cfg = inputs.CONFIGS[4]
    _check_product(oracle, cfg, "integer", None, strips="few")


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
