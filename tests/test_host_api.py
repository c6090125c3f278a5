"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol, and the
planner / memory / flop calls agree with the paper's formulas and with the oracle's tree walk."""
import math
import os
import re
import sys

import pytest

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sw_gemm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sw_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sw.EXPORTS)
    L = sw.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_model_words_equals_oracle_tree_walk(oracle):
    for n, levels, sched in [(256, 1, "B"), (4096, 3, "BBB"), (16384, 4, "DBBB"), (23520, 5, "BDBDB"),
                             (94080, 5, "DDDBB"), (94080, 5, "DDDDD"), (64, 2, "DB"), (64, 2, "BD")]:
        assert sw.sw_model_words(n, levels, sched) == oracle.peak_words(n, levels, sched) + 3 * n * n


def test_model_words_closed_forms():
    # Section 3.3.1: P * Mem_UM = 7 n^2 (7/4)^k - 4 n^2 ; Section 3.4.1: Mem_LM
    n, k = 4096, 3
    assert sw.sw_model_words(n, k, "BBB") == 7 * n * n * 7 ** k // 4 ** k - 4 * n * n
    n, l, k = 94080, 3, 2
    lm = sum(3 * n * n // 4 ** i for i in range(l)) + (7 * (n >> l) ** 2 * 7 ** k // 4 ** k - 4 * (n >> l) ** 2)
    assert sw.sw_model_words(n, l + k, "DDDBB") == lm
    # the paper-model footprint at n = 94080 worked out by hand from the two formulas above (GB, incl. A, B, C)
    for sched, gb in [("DDDDD", 283.16), ("DDDDB", 284.41), ("DDDBD", 289.39), ("DDDBB", 298.10)]:
        assert sw.sw_model_words(94080, 5, sched) * 8 / 1e9 == pytest.approx(gb, abs=0.01)


def test_flop_count_is_appendix_a_closed_form():
    for cfg in inputs.CONFIGS:
        n, L = cfg["n"], cfg["levels"]
        n0 = n >> L
        assert sw.sw_flop_count(n, L) == pytest.approx((2 * n0 + 4) * n0 * n0 * 7 ** L - 5 * n * n, rel=1e-14)
    with pytest.raises(sw.SwError):
        sw.sw_flop_count(100, 3)


def test_plan_memory_structure():
    # workspace really used: 21 half-size buffers per parent at a BFS step, 2 at a DFS step
    def elems(h):
        ld = (h + 15) // 16 * 16
        if ld >= 256 and ld % 256 == 0:
            ld += 16
        return (ld * h + 31) // 32 * 32
    assert sw.sw_plan_memory(256, 1, "B") == 21 * elems(128) * 8
    assert sw.sw_plan_memory(256, 1, "D") == 2 * elems(128) * 8
    assert sw.sw_plan_memory(1024, 2, "DB") == (2 * elems(512) + 21 * elems(256)) * 8
    assert sw.sw_plan_memory(1024, 2, "BD") == (21 * elems(512) + 2 * 7 * elems(256)) * 8
    assert sw.sw_plan_memory(1024, 2, None) == sw.sw_plan_memory(1024, 2, "DD")
    # two BFS steps in a row are fused: operands of the 49 grandchildren only, nothing for the level between
    assert sw.sw_plan_memory(1024, 2, "BB") == 3 * 49 * elems(256) * 8
    assert sw.sw_plan_memory(1024, 3, "BBB") == (21 * elems(512) + 3 * 49 * 7 * elems(128)) * 8   # odd run: top step alone
    assert sw.sw_plan_memory(1024, 3, "DBB") == (2 * elems(512) + 3 * 49 * elems(128)) * 8
    assert sw.sw_plan_memory(1024, 0, "") == 0
    # padding: 1001 -> 1008 with three padded copies
    assert sw.sw_plan_memory(1001, 3, "DDD") == sw.sw_plan_memory(1008, 3, "DDD") + 3 * elems(1008) * 8
    # never above the paper's model for the schedules used on the big configuration
    assert sw.sw_plan_memory(94080, 5, "DDDBB") < (sw.sw_model_words(94080, 5, "DDDBB") - 3 * 94080 ** 2) * 8


def test_planner_prefers_bfs_and_puts_dfs_first():
    assert sw.sw_plan_schedule(4096, 3, 10 ** 11) == "BBB"
    n, L = 94080, 5
    gib288 = 288 * 2 ** 30 - 3 * n * n * 8          # what is left of 288 GiB beside A, B, C
    s = sw.sw_plan_schedule(n, L, int(gib288 * 0.95))
    assert s == "DDDBB"
    assert sw.sw_plan_memory(n, L, s) <= gib288 * 0.95
    assert sw.sw_plan_schedule(n, L, int(288e9 - 3 * n * n * 8)) == "DDDBB"
    assert sw.sw_plan_schedule(n, L, int(50e9)) == "DDDDB"
    assert sw.sw_plan_schedule(n, L, int(47.5e9)) == "DDDDD"
    with pytest.raises(sw.SwError) as e:
        sw.sw_plan_schedule(n, L, 10 ** 9)
    assert e.value.code == sw.SW_ENOMEM
    # every schedule the planner returns fits its budget; a bigger budget never gives fewer BFS steps
    last = -1
    for budget in [10 ** 8, 10 ** 9, 4 * 10 ** 9, 10 ** 10, 10 ** 11, 10 ** 12]:
        s = sw.sw_plan_schedule(16384, 4, budget) if budget >= sw.sw_plan_memory(16384, 4, None) else None
        if s is not None:
            assert sw.sw_plan_memory(16384, 4, s) <= budget
            assert s.count("B") >= last
            last = s.count("B")
            assert "BD" not in s            # DFS steps first (Limited-Memory shape)


def test_plan_memory_with_peeling_at_every_level():
    def elems(h):
        ld = (h + 15) // 16 * 16
        if ld >= 256 and ld % 256 == 0:
            ld += 16
        return (ld * h + 31) // 32 * 32
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL_LEVELS)
    try:
        # extents halve rounding down: 1001 -> 500 -> 250 -> 125; no copies of the operands; a level with an odd inner
        # extent sets the peeled column of A and row of B aside (each rounded up to 32 doubles per problem)
        def side(e):
            return 2 * ((e + 31) // 32 * 32)
        assert sw.sw_plan_memory(1001, 3, "DDD") == (side(1000) + 2 * elems(500) + 2 * elems(250) + 2 * elems(125)) * 8
        assert sw.sw_plan_memory(1000, 3, "DDD") == (2 * elems(500) + 2 * elems(250) + 2 * elems(125)) * 8
        # a pair of BFS steps is one pass only where the level between them is even: 1001 -> 500 (even) fuses ...
        assert sw.sw_plan_memory(1001, 2, "BB") == (side(1000) + 3 * 49 * elems(250)) * 8
        # ... 1003 -> 501 (odd) does not: seven children of 501, each peeled again, then their 49 of 250
        assert sw.sw_plan_memory(1003, 2, "BB") == (side(1002) + 21 * elems(501) + 7 * side(500) + 21 * 7 * elems(250)) * 8
        assert sw.sw_plan_schedule(94097, 5, (290 << 30) - 3 * 94097 ** 2 * 8) == "DDDBB"
        with pytest.raises(sw.SwError):
            sw.sw_plan_memory(7, 3, "DDD")
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


def test_planner_picks_on_the_measured_sizes():
    """The planner's choice at the sizes where every step order was timed on the MI355X (profiles/step_orders.md):
    each pick below is the fastest measured order or within 0.3 % of it.  Only Limited-Memory shapes (DFS steps,
    then BFS steps; Section 3.4) are ever picked."""
    free = 290 << 30
    for n, L, want in [(4096, 3, "BBB"), (8192, 3, "DBB"), (8192, 4, "DBBB"), (16384, 4, "DDBB"), (23520, 5, "DBBBB"),
                       (32768, 4, "DDBB"), (47040, 4, "DDBB"), (94080, 5, "DDDBB")]:
        assert sw.sw_plan_schedule(n, L, free - 3 * n * n * 8) == want, (n, L)
    for n in (300, 1000, 5000, 20000, 70000):
        for L in range(1, 6):
            if (n >> L) < 16:
                continue
            for budget in (sw.sw_plan_memory(n, L, None), 10 ** 9, 10 ** 10, 10 ** 11):
                if budget < sw.sw_plan_memory(n, L, None):
                    continue
                s = sw.sw_plan_schedule(n, L, budget)
                assert "BD" not in s and sw.sw_plan_memory(n, L, s) <= budget
    # one stream: nothing runs beside the leaf products, the all-BFS order wins where it fits
    sw.sw_set_overlap(0)
    try:
        assert sw.sw_plan_schedule(16384, 4, free) == "BBBB"
    finally:
        sw.sw_set_overlap(1)
    # the model behind the choice: an order that does not fit has no time, one that fits has a positive one
    assert sw.sw_model_seconds_order(94080, 5, "DDBBB", int(50e9)) == -1.0
    assert 10.0 < sw.sw_model_seconds_order(94080, 5, "DDDBB", int(81e9)) < 16.0


def test_plan_workspace_spends_extra_memory_on_the_deepest_dfs_steps():
    def elems(h):
        ld = (h + 15) // 16 * 16
        if ld >= 256 and ld % 256 == 0:
            ld += 16
        return (ld * h + 31) // 32 * 32
    n, L, s = 1024, 3, "DDD"
    lean = sw.sw_plan_memory(n, L, s)
    assert lean == (2 * elems(512) + 2 * elems(256) + 2 * elems(128)) * 8
    assert sw.sw_plan_workspace(n, L, s, lean) == lean
    assert sw.sw_plan_workspace(n, L, s, lean + 13 * elems(128) * 8) == lean + 13 * elems(128) * 8     # deepest step rich
    assert sw.sw_plan_workspace(n, L, s, lean + 13 * elems(128) * 8 + 100) == lean + 13 * elems(128) * 8
    assert sw.sw_plan_workspace(n, L, s, 10 ** 10) == (15 * elems(512) + 15 * elems(256) + 15 * elems(128)) * 8
    assert sw.sw_plan_workspace(n, L, "BBB", 10 ** 10) == sw.sw_plan_memory(n, L, "BBB")               # nothing to upgrade
    with pytest.raises(sw.SwError) as e:
        sw.sw_plan_workspace(n, L, s, lean - 1)
    assert e.value.code == sw.SW_ENOMEM
    # configuration 5: the level-2 DFS step (49 nodes of 23520) is the one that fits in what 288 GiB leave
    n5 = 94080
    left = 288 * 2 ** 30 - 3 * n5 * n5 * 8 - 4 * 2 ** 30
    got = sw.sw_plan_workspace(n5, 5, "DDDBB", left)
    twice = 3 * 49 * elems(2940) * 8            # first a second set of the 49 leaf operands and products ...
    assert got == sw.sw_plan_memory(n5, 5, "DDDBB") + twice + 13 * elems(11760) * 8     # ... then the rich level-2 step
    sw.sw_set_overlap(False)
    try:
        assert sw.sw_plan_workspace(n5, 5, "DDDBB", left) == sw.sw_plan_memory(n5, 5, "DDDBB") + 13 * elems(11760) * 8
    finally:
        sw.sw_set_overlap(True)
    # a second set is pointless without a DFS step above (one launch) or when the leaves hang under a DFS step
    assert sw.sw_plan_workspace(4096, 3, "BBB", 10 ** 11) == sw.sw_plan_memory(4096, 3, "BBB")
    assert sw.sw_plan_workspace(1024, 2, "DB", 10 ** 10) == (15 * elems(512) + 2 * 21 * elems(256)) * 8


def test_peel_mode_needs_no_copies():
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL)
    try:
        assert sw.sw_plan_memory(1001, 3, "DDD") == sw.sw_plan_memory(1000, 3, "DDD")
        assert sw.sw_plan_memory(94097, 5, "DDDBB") == sw.sw_plan_memory(94080, 5, "DDDBB")
        assert sw.sw_plan_schedule(94097, 5, int(60e9)) == "DDDBB"
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)
    assert sw.sw_plan_memory(1001, 3, "DDD") > sw.sw_plan_memory(1008, 3, "DDD")
    with pytest.raises(sw.SwError):
        sw.sw_set_odd_mode(7)


def test_lm_dfs_step_formula():
    # l = max(0, ceil(log2(4 n / (P^(1/w0) sqrt(M)))))  (Section 3.4), checked inside its validity range
    w0 = math.log2(7)
    for n, P, M in [(94080, 49, 8e9 / 8), (94080, 343, 8e9 / 8), (94080, 2401, 8e9 / 8), (10 ** 6, 7, 1e9), (1000, 7, 1e9)]:
        expect = max(0, math.ceil(math.log2(4 * n / (P ** (1 / w0) * math.sqrt(M)))))
        assert sw.sw_lm_dfs_steps(n, P, M) == expect
    assert sw.sw_lm_dfs_steps(1000, 7, 1e9) == 0
    # the paper's own machine: n = 94080 on 49 nodes of 8 GB needs DFS steps, on 2401 nodes none
    assert sw.sw_lm_dfs_steps(94080, 49, 1e9) > sw.sw_lm_dfs_steps(94080, 2401, 1e9) == 0


def test_argument_errors_without_gpu():
    for args in [(-1, 0, None), (16, -1, None), (16, 17, None), (4, 3, None), (16, 2, "B"), (16, 2, "BX"), (300000, 1, "B")]:
        with pytest.raises(sw.SwError) as e:
            sw.sw_plan_memory(*args)
        assert e.value.code == sw.SW_EINVAL
        assert sw.sw_last_error() != ""
    with pytest.raises(sw.SwError):
        sw.sw_model_words(100, 3, "BBB")


# ---- other 2 x 2 block schemes (Section 6.6) ------------------------------------------------------------------

def test_bilinear_memory_and_flop_counts(oracle):
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import sw_bilinear

    def ws_mat_elems(h):     # the documented workspace rule: pitch a multiple of 16, never of 256; slots of 32
        ld = (h + 15) // 16 * 16
        ld += 16 if ld % 256 == 0 else 0
        return (ld * h + 31) // 32 * 32
    for scheme, q, oid in ((sw.SW_SCHEME_STRASSEN, 7, 0), (sw.SW_SCHEME_CLASSICAL, 8, 1)):
        n, levels = 1024, 3
        # BFS step: 3q half-size buffers per parent, the parents multiply by q; DFS step: 3 per parent
        want = 0
        live, size = 1, n
        for ch in "BDB":
            size //= 2
            want += (3 * q if ch == "B" else 3) * live * ws_mat_elems(size) * 8
            live *= q if ch == "B" else 1
        assert sw.sw_plan_memory_bilinear(n, levels, "BDB", scheme) == want
        assert sw.sw_plan_memory_bilinear(n, levels, None, scheme) == sw.sw_plan_memory_bilinear(n, levels, "DDD", scheme)
        # the operation count equals what the oracle actually performs
        m = 64
        A = inputs.matrix(m, 1, 0, "integer")
        sw_bilinear.reset_counters()
        sw_bilinear.gemm(A, A, 2, oid)
        c = sw_bilinear.counters()
        assert sw.sw_flop_count_bilinear(m, 2, scheme) == c["leaf_mul"] + c["leaf_add"] + c["block_add"]
    # 3 x 3 blocks: the step divides by three, q = 23 or 27 children; levels may carry different schemes
    for scheme, q, oid in ((sw.SW_SCHEME_LADERMAN, 23, 2), (sw.SW_SCHEME_CLASSICAL3, 27, 3)):
        n, levels = 1458, 3
        want, live, size = 0, 1, n
        for ch in "BDB":
            size //= 3
            want += (3 * q if ch == "B" else 3) * live * ws_mat_elems(size) * 8
            live *= q if ch == "B" else 1
        assert sw.sw_plan_memory_bilinear(n, levels, "BDB", scheme) == want
        assert sw.sw_plan_memory_bilinear(1000, 2, "DD", scheme) == sw.sw_plan_memory_bilinear(1008, 2, "DD", scheme) + 3 * ws_mat_elems(1008) * 8
        m = 54
        A = inputs.matrix(m, 1, 0, "integer")
        sw_bilinear.reset_counters()
        sw_bilinear.gemm(A, A, 2, oid)
        c = sw_bilinear.counters()
        assert sw.sw_flop_count_bilinear(m, 2, scheme) == c["leaf_mul"] + c["leaf_add"] + c["block_add"]
        assert sw.sw_flop_count_bilinear(m + 1, 2, scheme) == -1.0
    mixed = [sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_LADERMAN]
    assert sw.sw_plan_memory_bilinear_levels(600, "BD", mixed) == (21 * ws_mat_elems(300) + 3 * 7 * ws_mat_elems(100)) * 8
    assert sw.sw_plan_memory_bilinear_levels(600, "DB", mixed) == (3 * ws_mat_elems(300) + 3 * 23 * ws_mat_elems(100)) * 8
    assert sw.sw_plan_memory_bilinear_levels(601, "DB", mixed) == sw.sw_plan_memory_bilinear_levels(606, "DB", mixed) + 3 * ws_mat_elems(606) * 8
    with pytest.raises(sw.SwError):
        sw.sw_plan_memory_bilinear_levels(600, "DB", [sw.SW_SCHEME_STRASSEN, sw.SW_SCHEME_WINOGRAD])
    assert sw.sw_flop_count_bilinear(4096, 3, sw.SW_SCHEME_CLASSICAL) == 2.0 * 4096 ** 3 - 4096 ** 2
    assert sw.sw_flop_count_bilinear(4096, 3, sw.SW_SCHEME_WINOGRAD) == sw.sw_flop_count(4096, 3)
    assert sw.sw_plan_memory_bilinear(4096, 3, "BBB", sw.SW_SCHEME_WINOGRAD) == sw.sw_plan_memory(4096, 3, "BBB")
    with pytest.raises(sw.SwError):
        sw.sw_plan_memory_bilinear(64, 1, "B", 9)


def test_plan_levels_and_dgemm_memory():
    # depth model: classical for small products, five steps at the headline size (as measured), never a
    # depth no step order fits, and non-decreasing in n for a generous budget
    big = 250 << 30
    assert sw.sw_plan_levels(0, big) == 0 and sw.sw_plan_levels(512, big) == 0
    assert sw.sw_plan_levels(94080, 95 << 30) == 5
    assert sw.sw_plan_levels(94080, 0) == 0
    prev = 0
    for n in (1024, 4096, 16384, 32768, 65536, 131072):
        L = sw.sw_plan_levels(n, big)
        assert L >= prev
        prev = L
        assert sw.sw_plan_memory(n, L, None) <= big
    # dgemm workspace (the largest block shape it considers: the whole product, rounded down to multiples of
    # 2^levels): the recursion's own plus a temporary for C's block and one more per transposed operand
    def elems(rows, cols):
        ld = (cols + 15) // 16 * 16
        ld += 16 if ld >= 256 and ld % 256 == 0 else 0
        return (ld * rows + 31) // 32 * 32
    M, N, K, L = 5003, 3001, 4005, 3
    sm, sn, sk = 5000, 3000, 4000
    inner = sw.sw_plan_memory_rect(sm, sn, sk, L, "DBB")
    assert sw.sw_plan_memory_dgemm(0, 0, M, N, K, L, "DBB") == inner + 8 * elems(sm, sn)
    assert sw.sw_plan_memory_dgemm(1, 0, M, N, K, L, "DBB") == inner + 8 * (elems(sm, sn) + elems(sm, sk))
    assert sw.sw_plan_memory_dgemm(1, 1, M, N, K, L, "DBB") == inner + 8 * (elems(sm, sn) + elems(sm, sk) + elems(sk, sn))
    with pytest.raises(sw.SwError):
        sw.sw_plan_memory_dgemm(0, 0, 64, 64, 3, 2, "BB")


def test_rectangular_memory_formula():
    def elems(rows, cols):     # the documented workspace rule: pitch a multiple of 16, never of 256; slots of 32
        ld = (cols + 15) // 16 * 16
        ld += 16 if ld >= 256 and ld % 256 == 0 else 0
        return (ld * rows + 31) // 32 * 32
    M, N, K = 1024, 512, 2048
    # one BFS step: seven T (M/2 x K/2), seven S (K/2 x N/2), seven Q (M/2 x N/2)
    assert sw.sw_plan_memory_rect(M, N, K, 1, "B") == 7 * 8 * (elems(512, 1024) + elems(1024, 256) + elems(512, 256))
    # one DFS step: a temporary that holds a T or a Q, and one for an S
    assert sw.sw_plan_memory_rect(M, N, K, 1, "D") == 8 * (max(elems(512, 1024), elems(512, 256)) + elems(1024, 256))
    # a cube is the square product
    assert sw.sw_plan_memory_rect(4096, 4096, 4096, 3, "DBB") == sw.sw_plan_memory(4096, 3, "DBB")
    # padding: three copies at the padded extents
    base = sw.sw_plan_memory_rect(104, 72, 40, 3, "DDD")
    assert sw.sw_plan_memory_rect(100, 70, 33, 3, "DDD") == base + 8 * (elems(104, 40) + elems(40, 72) + elems(104, 72))
    with pytest.raises(sw.SwError):
        sw.sw_plan_memory_rect(64, 64, 3, 2, "BB")


def test_leading_dimensions_beyond_the_product_kernels_reach_are_refused():
    """The product kernel addresses a tile with 32-bit byte offsets per lane (127 rows of A, 15 rows of B from a
    64-bit base): leading dimensions that would wrap them are an argument error before anything is launched.
    No device memory is touched: the pointers are made up and never dereferenced."""
    import ctypes
    L = sw.lib()
    p = lambda k: ctypes.c_void_p(k << 40)
    lda_ok, lda_bad = 4227329, 4227330           # (127 lda + 16) * 8 < 2^32
    ldb_ok, ldb_bad = 35791385, 35791386         # (15 ldb + 128) * 8 < 2^32
    assert (127 * lda_ok + 16) * 8 < 2 ** 32 <= (127 * lda_bad + 16) * 8
    assert (15 * ldb_ok + 128) * 8 < 2 ** 32 <= (15 * ldb_bad + 128) * 8
    n = 256
    for lda, ldb in ((lda_bad, n), (n, ldb_bad), (1 << 33, n)):
        assert L.sw_leaf_gemm(n, 1, p(1), lda, 0, p(2), ldb, 0, p(3), n, 0, None) == sw.SW_EINVAL
        assert "32-bit" in sw.sw_last_error()
        assert L.sw_gemm_classical(n, n, n, p(1), lda, p(2), ldb, p(3), n, 0, None) == sw.SW_EINVAL
        assert L.sw_gemm_ex(n, p(1), lda, p(2), ldb, p(3), n, 1, b"D", p(4), 1 << 30, None) == sw.SW_EINVAL
        assert "32-bit" in sw.sw_last_error()
        assert L.sw_gemm_rect(n, n, n, p(1), lda, p(2), ldb, p(3), n, 0, b"", None, 0, None) == sw.SW_EINVAL
        assert L.sw_gemm_static(n, p(1), lda, p(2), ldb, p(3), n, 1, b"D", None) == sw.SW_EINVAL
    sw.sw_set_workspace(None)
    assert L.sw_dgemm(0, 0, n, n, n, 1.0, p(1), lda_bad, p(2), n, 0.0, p(3), n, 0, b"") == sw.SW_EINVAL
    assert L.sw_dgemm(0, 0, n, n, n, 1.0, p(1), n, p(2), ldb_bad, 0.0, p(3), n, 0, b"") == sw.SW_EINVAL
    # the record-only run takes the same path and accepts the largest pitches that fit
    assert L.sw_trace_gemm(n, n, n, lda_ok, ldb_ok, n, 1, b"D", 1 << 30, 1, 0, -1, None, 0) > 0
    assert L.sw_trace_gemm(n, n, n, lda_bad, ldb_ok, n, 1, b"D", 1 << 30, 1, 0, -1, None, 0) == sw.SW_EINVAL


def test_static_scratch_limit_is_checked_on_the_host():
    """sw_gemm_static refuses, before it touches the device, a product whose workspace exceeds its array."""
    import ctypes
    L = sw.lib()
    p = lambda k: ctypes.c_void_p(k << 40)
    assert sw.sw_plan_memory(8192, 2, "DD") > sw.SW_STATIC_SCRATCH_BYTES
    assert L.sw_gemm_static(8192, p(1), 8192, p(2), 8192, p(3), 8192, 2, b"DD", None) == sw.SW_ENOMEM
    assert "static scratch" in sw.sw_last_error()
    header = open(os.path.join(ROOT, "include", "sw_gemm.h")).read()
    assert re.search(r"#define SW_STATIC_SCRATCH_BYTES \(128 \* 1024 \* 1024\)", header)
    assert sw.SW_STATIC_SCRATCH_BYTES == 128 * 1024 * 1024
