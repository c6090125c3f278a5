"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on seeded inputs.

Bar: fp64 results within max|C - C_ref| <= 1e-10 * n * max|A| * max|B| (the build's stated tolerance, whose
form is the norm-wise bound of Section 6.1); integer-valued inputs, for which every intermediate of the
recursion is an exactly representable integer, must agree BIT FOR BIT with the oracle and with the exact
product; results must not depend on the BFS/DFS order at all.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def tol(n, A, B):
    return 1e-10 * n * float(np.max(np.abs(A))) * float(np.max(np.abs(B)))


def run(A, B, levels, schedule):
    n = A.shape[0]
    dA = torch.from_numpy(A).to(DEV)
    dB = torch.from_numpy(B).to(DEV)
    C = sw.matmul(dA, dB, levels, schedule)
    torch.cuda.synchronize()
    assert torch.equal(dA.cpu(), torch.from_numpy(A)) and torch.equal(dB.cpu(), torch.from_numpy(B)), "inputs changed"
    return C.cpu().numpy()


# ---- the generator is the same on host and device --------------------------------------------------------------

@pytest.mark.parametrize("dist", ["uniform", "rowscaled", "integer"])
def test_device_generator_matches_host(dist):
    n = 333
    for which in (0, 1):
        t = torch.empty((n, n), dtype=torch.float64, device=DEV)
        inputs.fill_device(t, n, 42, which, dist)
        torch.cuda.synchronize()
        assert np.array_equal(t.cpu().numpy(), inputs.matrix(n, 42, which, dist))


# ---- leaf products ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("m,batch,ldpad", [(1, 1, 0), (16, 3, 0), (100, 2, 0), (128, 1, 0), (129, 2, 1),
                                           (255, 1, 1), (256, 2, 0), (300, 3, 4), (735, 2, 1), (514, 1, 2),
                                           (735, 2, 3), (129, 3, 3), (5, 2, 3), (143, 1, 17)])
def test_leaf_gemm_against_classical_oracle(oracle, m, batch, ldpad):
    ld = m + ldpad
    stride = ld * m + (7 if ldpad == 1 else 0)   # ldpad 1: odd stride, the 8-byte load path; odd m with an
    #                                              even padded pitch and stride: 16-byte loads that straddle the edge
    hA = [inputs.matrix(m, 3 + b, 0, "uniform") for b in range(batch)]
    hB = [inputs.matrix(m, 3 + b, 1, "uniform") for b in range(batch)]
    A = torch.zeros(batch * stride, dtype=torch.float64, device=DEV)
    B = torch.zeros(batch * stride, dtype=torch.float64, device=DEV)
    C = torch.full((batch * stride,), float("nan"), dtype=torch.float64, device=DEV)
    for b in range(batch):
        A[b * stride: b * stride + ld * m].view(m, ld)[:, :m] = torch.from_numpy(hA[b]).to(DEV)
        B[b * stride: b * stride + ld * m].view(m, ld)[:, :m] = torch.from_numpy(hB[b]).to(DEV)
    sw.sw_leaf_gemm(m, batch, A, ld, stride, B, ld, stride, C, ld, stride)
    torch.cuda.synchronize()
    for b in range(batch):
        got = C[b * stride: b * stride + ld * m].view(m, ld)[:, :m].cpu().numpy()
        ref = oracle.naive(hA[b], hB[b])
        assert np.max(np.abs(got - ref)) <= tol(m, hA[b], hB[b])
        assert np.max(np.abs(got - ref)) <= 4 * m * np.finfo(float).eps   # classical: a few ulps per term
        pad = C[b * stride: b * stride + ld * m].view(m, ld)[:, m:]
        assert torch.isnan(pad).all(), "wrote outside the m x m result"


def test_leaf_gemm_integer_exact(oracle):
    for m in (64, 200, 735):
        hA = inputs.matrix(m, 1, 0, "integer")
        hB = inputs.matrix(m, 1, 1, "integer")
        A, B = torch.from_numpy(hA).to(DEV), torch.from_numpy(hB).to(DEV)
        C = torch.empty_like(A)
        sw.sw_leaf_gemm(m, 1, A, m, 0, B, m, 0, C, m, 0)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), oracle.naive(hA, hB))
        assert np.array_equal(C.cpu().numpy(), (hA.astype(np.int64) @ hB.astype(np.int64)).astype(np.float64))


# ---- one BFS step's additions, bit for bit (additions are exactly rounded, association as in Appendix A) -----------

@pytest.mark.parametrize("h,live", [(8, 1), (97, 3), (128, 7), (735, 2), (300, 1)])
def test_pre_and_post_add_bitwise(h, live):
    n = 2 * h
    ld = (h + 15) // 16 * 16
    cs = ld * h + 32
    P = torch.from_numpy(np.stack([inputs.matrix(n, 50 + p, 0, "uniform") for p in range(live)])).to(DEV)
    hP = P.cpu().numpy()
    q = lambda M, i, j: M[:, i * h:(i + 1) * h, j * h:(j + 1) * h]
    a11, a12, a21, a22 = q(hP, 0, 0), q(hP, 0, 1), q(hP, 1, 0), q(hP, 1, 1)
    for side in (0, 1):
        out = torch.full((live * 7 * cs,), float("nan"), dtype=torch.float64, device=DEV)
        sw.sw_pre_add(side, P, n, n * n, live, h, out, ld, cs)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(live, 7, cs)[:, :, :ld * h].reshape(live, 7, h, ld)
        assert np.isnan(got[..., h:]).all()
        got = got[..., :h]
        if side == 0:
            t2 = a21 + a22; t3 = t2 - a11; t4 = a11 - a21; t5 = a12 - t3
            want = [a11, a12, t2, t3, t4, t5, a22]
        else:
            s2 = a12 - a11; s3 = a22 - s2; s4 = a22 - a12; s6 = s3 - a21
            want = [a11, a21, s2, s3, s4, a22, s6]
        for j in range(7):
            assert np.array_equal(got[:, j], want[j]), (side, j)
    # post-additions
    Q = torch.from_numpy(np.stack([inputs.matrix(h, 80 + i, 1, "uniform") for i in range(live * 7)])).to(DEV)
    hQ = Q.cpu().numpy().reshape(live, 7, h, h)
    Cp = torch.full((live, n, n), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_post_add(Q, h, h * h, live, h, Cp, n, n * n)
    torch.cuda.synchronize()
    got = Cp.cpu().numpy()
    u1 = hQ[:, 0] + hQ[:, 3]; u2 = u1 + hQ[:, 4]; u3 = u1 + hQ[:, 2]
    assert np.array_equal(q(got, 0, 0), hQ[:, 0] + hQ[:, 1])
    assert np.array_equal(q(got, 0, 1), u3 + hQ[:, 5])
    assert np.array_equal(q(got, 1, 0), u2 - hQ[:, 6])
    assert np.array_equal(q(got, 1, 1), u2 + hQ[:, 2])


@pytest.mark.parametrize("m,live", [(5, 1), (64, 2), (147, 3), (200, 1)])
def test_fused_two_step_additions_equal_two_single_steps(m, live):
    # sw_pre_add2 / sw_post_add2 must give the very bits of two sw_pre_add / sw_post_add passes
    n, h = 4 * m, 2 * m
    ld = lambda x: (x + 15) // 16 * 16
    P = torch.from_numpy(np.stack([inputs.matrix(n, 70 + p, 0, "uniform") for p in range(live)])).to(DEV)
    for side in (0, 1):
        mid = torch.empty((live * 7, h, ld(h)), dtype=torch.float64, device=DEV)
        sw.sw_pre_add(side, P, n, n * n, live, h, mid, ld(h), h * ld(h))
        two = torch.full((live * 49, m, ld(m)), float("nan"), dtype=torch.float64, device=DEV)
        sw.sw_pre_add(side, mid, ld(h), h * ld(h), live * 7, m, two, ld(m), m * ld(m))
        one = torch.full((live * 49, m, ld(m)), float("nan"), dtype=torch.float64, device=DEV)
        sw.sw_pre_add2(side, P, n, n * n, live, m, one, ld(m), m * ld(m))
        torch.cuda.synchronize()
        assert torch.equal(one[:, :, :m], two[:, :, :m]), side
        assert torch.isnan(one[:, :, m:]).all()
    Q = torch.from_numpy(np.stack([inputs.matrix(m, 300 + i, 1, "uniform") for i in range(live * 49)])).to(DEV)
    mid = torch.empty((live * 7, h, h), dtype=torch.float64, device=DEV)
    sw.sw_post_add(Q, m, m * m, live * 7, m, mid, h, h * h)
    two = torch.empty((live, n, n), dtype=torch.float64, device=DEV)
    sw.sw_post_add(mid, h, h * h, live, h, two, n, n * n)
    one = torch.full((live, n, n), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_post_add2(Q, m, m * m, live, m, one, n, n * n)
    torch.cuda.synchronize()
    assert torch.equal(one, two)


def test_pad_copy_and_crop():
    src = torch.from_numpy(inputs.matrix(37, 1, 0, "uniform")).to(DEV)
    dst = torch.full((40, 48), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_pad_copy(src, 37, 37, 37, dst, 48, 40, 40)
    torch.cuda.synchronize()
    d = dst.cpu().numpy()
    assert np.array_equal(d[:37, :37], src.cpu().numpy())
    assert (d[37:40, :40] == 0).all() and (d[:40, 37:40] == 0).all() and np.isnan(d[:, 40:]).all()
    back = torch.empty((37, 37), dtype=torch.float64, device=DEV)
    sw.sw_pad_copy(dst, 48, 40, 40, back, 37, 37, 37)
    torch.cuda.synchronize()
    assert torch.equal(back, src)


# ---- the whole product against the oracle ---------------------------------------------------------------------------

CASES = [
    (256, 1, ["B", "D"], "uniform"),            # configuration 1
    (64, 2, ["BB", "DD"], "uniform"),
    (512, 2, ["BB", "BD", "DB", "DD"], "normal"),
    (1000, 3, ["BBB", "DBD", "BDB", "DDD"], "rowscaled"),     # leaf 125: odd, several tiles, ragged
    (1001, 3, ["DBB", "BDD"], "uniform"),                     # padded to 1008, leaf 126
    (777, 2, ["BB", "DB"], "uniform"),                        # padded to 780, leaf 195
    (2940, 2, ["DB", "BB"], "uniform"),                       # leaf 735 as in configuration 4
    (96, 5, ["BDBDB", "DDDDD", "BBBBB", "DBBBB", "BBDBB"], "uniform"),   # leaf 3; odd and even runs of BFS steps
    (1200, 4, ["BBBB", "DBBB", "DDBB", "BBDB"], "uniform"),   # leaf 75; fused pairs of BFS steps
    (300, 0, [""], "uniform"),                                # no Strassen step at all
    (1, 0, [""], "uniform"),
]


@pytest.mark.parametrize("n,levels,schedules,dist", CASES)
def test_product_matches_oracle(oracle, n, levels, schedules, dist):
    A = inputs.matrix(n, 1000 + n, 0, dist)
    B = inputs.matrix(n, 1000 + n, 1, dist)
    ref = oracle.gemm(A, B, levels)
    first = None
    for s in schedules:
        C = run(A, B, levels, s)
        err = float(np.max(np.abs(C - ref)))
        assert err <= tol(n, A, B), (s, err)
        if first is None:
            first = C
        else:
            assert np.array_equal(C, first), f"result depends on the step order ({schedules[0]} vs {s})"
    # integer-valued inputs: exact, equal to the oracle and to the integer product, whatever the order
    Ai = inputs.matrix(n, 2000 + n, 0, "integer")
    Bi = inputs.matrix(n, 2000 + n, 1, "integer")
    exact = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64)
    assert np.array_equal(oracle.gemm(Ai, Bi, levels), exact)
    for s in schedules:
        assert np.array_equal(run(Ai, Bi, levels, s), exact), s


@pytest.mark.parametrize("M,N,K,acc", [(1, 1, 1, False), (130, 5, 70, False), (5, 130, 257, True), (300, 300, 3, True),
                                        (257, 129, 64, False), (17, 1000, 1000, False), (640, 31, 641, True)])
def test_classical_product_general_shapes(oracle, M, N, K, acc):
    # the oracle's classical product is square: embed the rectangular operands in zero-padded squares
    d = max(M, N, K)
    A = np.zeros((d, d)); B = np.zeros((d, d))
    A[:M, :K] = inputs.matrix(d, 31, 0, "uniform")[:M, :K]
    B[:K, :N] = inputs.matrix(d, 31, 1, "uniform")[:K, :N]
    ref = oracle.naive(A, B)[:M, :N]
    C0 = inputs.matrix(d, 32, 0, "uniform")[:M, :N].copy()
    dA = torch.from_numpy(A[:M, :K].copy()).to(DEV)
    dB = torch.from_numpy(B[:K, :N].copy()).to(DEV)
    dC = torch.from_numpy(C0).to(DEV)
    sw.sw_gemm_classical(M, N, K, dA, K, dB, N, dC, N, accumulate=acc)
    torch.cuda.synchronize()
    want = ref + C0 if acc else ref
    assert np.max(np.abs(dC.cpu().numpy() - want)) <= 1e-10 * max(K, 1)
    assert np.max(np.abs(dC.cpu().numpy() - want)) <= 8 * K * np.finfo(float).eps


@pytest.mark.parametrize("n,levels,schedules", [(1001, 3, ["DBB", "BDD"]), (777, 2, ["BB", "DB"]), (263, 3, ["BBB"]),
                                                (97, 5, ["DDDBB"]), (1030, 1, ["B", "D"])])
def test_peeling_matches_oracle(oracle, n, levels, schedules):
    A = inputs.matrix(n, 4000 + n, 0, "uniform")
    B = inputs.matrix(n, 4000 + n, 1, "uniform")
    Ai = inputs.matrix(n, 5000 + n, 0, "integer")
    Bi = inputs.matrix(n, 5000 + n, 1, "integer")
    ref = oracle.gemm(A, B, levels)                 # the oracle pads; both approximate the same product
    exact = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64)
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL)
    try:
        assert sw.sw_plan_memory(n, levels, schedules[0]) == sw.sw_plan_memory(n - n % 2 ** levels, levels, schedules[0])
        for s in schedules:
            assert float(np.max(np.abs(run(A, B, levels, s) - ref))) <= tol(n, A, B)
            assert np.array_equal(run(Ai, Bi, levels, s), exact), s
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


@pytest.mark.parametrize("n,levels", [(3, 1), (97, 4), (127, 6), (263, 3), (777, 2), (1001, 3), (1000, 3), (1471, 2), (1470, 4)])
def test_peeling_at_every_odd_level_matches_oracle(oracle, n, levels):
    """SW_ODD_PEEL_LEVELS against the oracle's recursion with the same peeling (sizes odd at one, several or all
    levels, and even ones): within the tolerance on real inputs, the exact product on integer-valued ones, the same
    bits for every step order, no workspace beyond what the halved (rounded-down) extents need, and rows beyond n
    of a wider C untouched."""
    A = inputs.matrix(n, 7000 + n, 0, "uniform")
    B = inputs.matrix(n, 7000 + n, 1, "rowscaled")
    Ai = inputs.matrix(n, 8000 + n, 0, "integer")
    Bi = inputs.matrix(n, 8000 + n, 1, "integer")
    ref = oracle.gemm_peel(A, B, levels)
    exact = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64)
    orders = ["".join("B" if (mask >> i) & 1 else "D" for i in range(levels)) for mask in range(1 << levels)]
    if len(orders) > 8:
        orders = orders[:2] + orders[len(orders) // 2 - 1:len(orders) // 2 + 2] + orders[-3:]
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL_LEVELS)
    try:
        assert sw.sw_plan_memory(n, levels, "D" * levels) <= sw.sw_plan_memory(n + 2 ** levels, levels, "D" * levels)
        first = None
        for s in orders:
            got = run(A, B, levels, s)
            assert float(np.max(np.abs(got - ref))) <= tol(n, A, B), s
            if first is None:
                first = got
            assert np.array_equal(got, first), s
            assert np.array_equal(run(Ai, Bi, levels, s), exact), s
        # views with leading dimensions: nothing is written beside the n columns
        ld = n + 5
        big = [torch.zeros((n, ld), dtype=torch.float64, device=DEV) for _ in range(2)]
        big[0][:, :n] = torch.from_numpy(Ai).to(DEV)
        big[1][:, :n] = torch.from_numpy(Bi).to(DEV)
        Cb = torch.full((n, ld), -7.0, dtype=torch.float64, device=DEV)
        ws = torch.empty(max(256, sw.sw_plan_memory(n, levels, orders[-1])), dtype=torch.uint8, device=DEV)
        sw.sw_gemm_ex(n, big[0], ld, big[1], ld, Cb, ld, levels, orders[-1], ws)
        torch.cuda.synchronize()
        assert np.array_equal(Cb[:, :n].cpu().numpy(), exact) and bool((Cb[:, n:] == -7.0).all())
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


def test_peeling_at_every_odd_level_on_rectangular_products():
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL_LEVELS)
    try:
        for (M, N, K, levels, order) in [(301, 515, 777, 3, "DBD"), (1001, 64, 333, 2, "BB"), (97, 97, 1030, 4, "DDBB"), (640, 641, 642, 3, "BDB"),
                                     (65, 131, 4099, 1, "B"), (4101, 35, 67, 1, "D"), (35, 4611, 2049, 2, "BB")]:   # one-wide kernels: several LDS chunks of the inner index, many row and column blocks
            g = torch.Generator(device=DEV).manual_seed(M + N)
            A = torch.randint(-8, 9, (M, K), generator=g, device=DEV, dtype=torch.int32).to(torch.float64)
            B = torch.randint(-8, 9, (K, N), generator=g, device=DEV, dtype=torch.int32).to(torch.float64)
            C = torch.full((M, N), float("nan"), dtype=torch.float64, device=DEV)
            ws = torch.empty(max(256, sw.sw_plan_memory_rect(M, N, K, levels, order)), dtype=torch.uint8, device=DEV)
            sw.sw_gemm_rect(M, N, K, A, K, B, N, C, N, levels, order, ws)
            torch.cuda.synchronize()
            assert torch.equal(C, A @ B), (M, N, K, order)
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


@pytest.mark.parametrize("n,levels,sched", [(512, 2, "DD"), (1000, 3, "DBD"), (1200, 4, "DDBB"), (96, 5, "BDBDB"), (777, 2, "DB")])
def test_dfs_steps_with_bfs_storage_give_the_same_bits(oracle, n, levels, sched):
    # with workspace beyond the minimum, DFS steps keep T, S, Q and use the one-pass addition kernels
    A = inputs.matrix(n, 6000 + n, 0, "uniform")
    B = inputs.matrix(n, 6000 + n, 1, "uniform")
    lean = run(A, B, levels, sched)
    assert float(np.max(np.abs(lean - oracle.gemm(A, B, levels)))) <= tol(n, A, B)
    need = sw.sw_plan_memory(n, levels, sched)
    full = sw.sw_plan_workspace(n, levels, sched, 10 ** 11)
    assert full > need
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    results = []
    for nbytes in sorted({full, (need + full) // 2 // 256 * 256}):
        C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        sw.sw_profile_enable(True)
        sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, sched, ws)
        torch.cuda.synchronize()
        prof = sw.sw_profile_read()
        sw.sw_profile_enable(False)
        assert np.array_equal(C.cpu().numpy(), lean), nbytes
        results.append(prof["dfs_add"]["launches"])
    assert results[-1] == 0          # every DFS step in its rich form: no element-wise DFS kernels left


def test_configuration_2_full_against_oracle(oracle):
    cfg = inputs.CONFIGS[1]
    n, levels = cfg["n"], cfg["levels"]
    A, B = inputs.pair(cfg)
    ref = oracle.gemm(A, B, levels)
    C = run(A, B, levels, cfg["schedule"])
    assert float(np.max(np.abs(C - ref))) <= tol(n, A, B)
    assert np.array_equal(C, run(A, B, levels, "DBD"))


def test_planner_choice_runs_and_library_state_calls(oracle):
    n, levels = 640, 3
    A = inputs.matrix(n, 5, 0, "uniform")
    B = inputs.matrix(n, 5, 1, "uniform")
    ref = oracle.gemm(A, B, levels)
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.empty_like(dA)
    for budget, expect in [(sw.sw_plan_memory(n, levels, "DDD"), "DDD"), (sw.sw_plan_memory(n, levels, "DDB"), "DDB"),
                           (10 ** 9, "BBB")]:
        assert sw.sw_plan_schedule(n, levels, budget) == expect
        ws = torch.empty(budget, dtype=torch.uint8, device=DEV)
        sw.sw_set_workspace(ws)
        sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
        C.fill_(float("nan"))
        sw.sw_gemm(n, dA, dB, C, levels, None)          # planner picks for this workspace
        torch.cuda.synchronize()
        assert float(np.max(np.abs(C.cpu().numpy() - ref))) <= tol(n, A, B)
        sw.sw_set_workspace(None)
    sw.sw_set_stream(0)


def test_side_stream_and_profile_record(oracle):
    n, levels = 512, 2
    A = inputs.matrix(n, 8, 0, "uniform")
    B = inputs.matrix(n, 8, 1, "uniform")
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.empty_like(dA)
    ws = torch.empty(sw.sw_plan_memory(n, levels, "DB"), dtype=torch.uint8, device=DEV)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    sw.sw_profile_enable(True)
    with torch.cuda.stream(st):
        sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, "DB", ws)
    st.synchronize()
    prof = sw.sw_profile_read()
    sw.sw_profile_enable(False)
    assert float(np.max(np.abs(C.cpu().numpy() - oracle.gemm(A, B, levels)))) <= tol(n, A, B)
    assert prof["leaf_gemm"]["launches"] == 7 and prof["leaf_gemm"]["work"] == 49 * 2.0 * 128 ** 3
    assert prof["pre_add"]["launches"] == 14 and prof["post_add"]["launches"] == 7
    assert prof["dfs_add"]["launches"] == 8 and prof["pad"]["launches"] == 0
    assert all(v["ms"] > 0 for k, v in prof.items() if v["launches"])


@pytest.mark.parametrize("n,levels,sched", [(1200, 4, "DDBB"), (1000, 3, "DBD"), (768, 3, "DDB"), (1536, 3, "DBB"), (640, 2, "DD")])
def test_three_stream_overlap_gives_the_same_bits_as_one_stream(oracle, n, levels, sched):
    # additions and leaf products on separate streams, ordered by tracked address ranges: any missed
    # dependency would show as a difference from the one-stream result (or between repeated runs)
    A = inputs.matrix(n, 7000 + n, 0, "uniform")
    B = inputs.matrix(n, 7000 + n, 1, "uniform")
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    results = {}
    try:
        for overlap in (False, True):
            sw.sw_set_overlap(overlap)
            for budget in (sw.sw_plan_memory(n, levels, sched), 10 ** 11):       # minimum, and everything it can use
                ws = torch.empty(sw.sw_plan_workspace(n, levels, sched, budget), dtype=torch.uint8, device=DEV)
                for rep in range(3):
                    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
                    ws.random_(0, 255)
                    sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, sched, ws)
                    torch.cuda.synchronize()
                    results[(overlap, budget, rep)] = C.cpu().numpy()
    finally:
        sw.sw_set_overlap(True)
    first = results[(False, sw.sw_plan_memory(n, levels, sched), 0)]
    assert float(np.max(np.abs(first - oracle.gemm(A, B, levels)))) <= tol(n, A, B)
    for key, val in results.items():
        assert np.array_equal(val, first), key


def test_two_host_threads_with_distinct_workspaces_and_streams():
    """Two host threads inside sw_gemm_ex at once (ctypes drops the interpreter lock during the call), each with its
    own operands, workspace and stream, many times over: every call takes its own internal streams and events, so
    the results are the ones each thread gets alone (exact products of integer-valued inputs)."""
    import threading
    jobs = []
    for k, (n, levels, sched) in enumerate([(1536, 3, "DDB"), (1280, 3, "DBB")]):
        A, B = inputs.device_pair(dict(n=n, seed=60 + k, dist="integer"), DEV)
        C = torch.empty((n, n), dtype=torch.float64, device=DEV)
        ws = torch.empty(sw.sw_plan_workspace(n, levels, sched, 1 << 33), dtype=torch.uint8, device=DEV)
        jobs.append(dict(n=n, levels=levels, sched=sched, A=A, B=B, C=C, ws=ws, stream=torch.cuda.Stream(), want=A @ B, bad=[]))
    torch.cuda.synchronize()
    go = threading.Barrier(2)

    def work(j):
        go.wait()
        for rep in range(12):
            j["C"].fill_(float("nan"))
            torch.cuda.synchronize()
            sw.sw_gemm_ex(j["n"], j["A"], j["n"], j["B"], j["n"], j["C"], j["n"], j["levels"], j["sched"], j["ws"], j["stream"].cuda_stream)
            j["stream"].synchronize()
            if not torch.equal(j["C"], j["want"]):
                j["bad"].append(rep)

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert [j["bad"] for j in jobs] == [[], []]


def test_product_can_be_captured_in_a_hip_graph_and_replayed(oracle):
    # the library allocates nothing, records no memset and never synchronises, so a caller may capture it;
    # every replay, with eager work of the program in between, must reproduce the eager result
    n, levels, sched = 320, 3, "DBB"
    A = inputs.matrix(n, 61, 0, "uniform")
    B = inputs.matrix(n, 61, 1, "uniform")
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    C = torch.empty_like(dA)
    ws = torch.empty(sw.sw_plan_workspace(n, levels, sched, 10 ** 9), dtype=torch.uint8, device=DEV)
    sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, sched, ws)
    torch.cuda.synchronize()
    eager = C.clone()
    assert float(np.max(np.abs(eager.cpu().numpy() - oracle.gemm(A, B, levels)))) <= tol(n, A, B)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, sched, ws)       # launches go to the capturing stream
    other = torch.from_numpy(inputs.matrix(n, 62, 0, "uniform")).to(DEV)
    for rep in range(4):
        C.fill_(float("nan"))
        ws.random_(0, 255)                                            # workspace contents must not matter
        scratch = other @ other                                       # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, eager), rep
        assert torch.isfinite(scratch).all()


def test_argument_errors_on_device():
    n = 64
    A = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    B = torch.zeros_like(A)
    C = torch.zeros_like(A)
    ws = torch.empty(sw.sw_plan_memory(n, 2, "BB"), dtype=torch.uint8, device=DEV)
    cases = [
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, A, n, 2, "BB", ws), sw.SW_EINVAL),       # C aliases A
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 2, "B", ws), sw.SW_EINVAL),        # schedule too short
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 2, "BQ", ws), sw.SW_EINVAL),
        (lambda: sw.sw_gemm_ex(n, A, n - 1, B, n, C, n, 2, "BB", ws), sw.SW_EINVAL),   # ld < n
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 7, "BBBBBBB", ws), sw.SW_EINVAL),  # 2^levels > n
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 2, "BB", ws[:1024]), sw.SW_ENOMEM),
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 2, "BB", None), sw.SW_ENOMEM),
        (lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, 2, None, ws[:256]), sw.SW_ENOMEM),  # planner: nothing fits
    ]
    for call, code in cases:
        with pytest.raises(sw.SwError) as e:
            call()
        assert e.value.code == code
    # n = 0 is a no-op
    Z = torch.zeros((0, 0), dtype=torch.float64, device=DEV)
    assert sw.lib().sw_gemm_ex(0, None, 0, None, 0, None, 0, 0, b"", None, 0, None) == sw.SW_OK
    assert Z.numel() == 0


# ---- a seeded sweep over sizes, depths, step orders, odd-size modes, executors and workspace sizes ------------------

def test_seeded_sweep_of_small_products_is_exact(oracle):
    """Forty seeded combinations nobody picked by hand: integer-valued operands, so the product must equal the
    exact integer product bit for bit whatever the size (odd ones included), depth, step order, odd-size mode
    (pad or peel), executor (one stream or three) and workspace (the minimum, or room for the second set of
    leaf-side buffers and the richer DFS steps)."""
    rng = np.random.default_rng(20240229)
    try:
        for case in range(40):
            levels = int(rng.integers(0, 5))
            n = int(rng.integers(max(1 << levels, 1), 700))
            schedule = "".join(rng.choice(["B", "D"]) for _ in range(levels))
            peel = bool(rng.integers(0, 2))
            overlap = bool(rng.integers(0, 2))
            roomy = bool(rng.integers(0, 2))
            sw.sw_set_odd_mode(sw.SW_ODD_PEEL if peel else sw.SW_ODD_PAD)
            sw.sw_set_overlap(overlap)
            A = inputs.matrix(n, 3000 + case, 0, "integer")
            B = inputs.matrix(n, 3000 + case, 1, "integer")
            need = sw.sw_plan_memory(n, levels, schedule)
            if roomy:
                need = sw.sw_plan_workspace(n, levels, schedule, need * 4 + (1 << 20))
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
            dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
            C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
            sw.sw_gemm_ex(n, dA, n, dB, n, C, n, levels, schedule, ws)
            torch.cuda.synchronize()
            exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
            assert np.array_equal(C.cpu().numpy(), exact), (case, n, levels, schedule, peel, overlap, roomy)
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)
        sw.sw_set_overlap(True)
