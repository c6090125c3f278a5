"""The executor's three-stream ordering, proved on the host.

`sw_trace_gemm` runs the executor without launching anything and writes down every kernel (with the memory its
launch arguments say it touches), every event record, every stream wait and every workspace buffer.  The checker
below knows nothing of the library's dependency tracker: it replays the record with the semantics of HIP streams
and events (a stream runs its kernels in order; a wait orders the waiting stream's LATER kernels after everything
the event's stream had been ordered after when the event was last recorded) using vector clocks, and reports

  * every pair of kernels on different streams that touch a common element, at least one of them writing,
    with no chain of waits between them (read-after-write, write-after-read, write-after-write);
  * every workspace buffer taken while overlapping a live one or reaching beyond the workspace, and every kernel
    that touches workspace memory outside the buffers live at its submission.

The planted-mistake tests withhold one declared range from the tracker (the kernel still touches it) and expect
the checker to object.
"""
import numpy as np
import pytest

from paper_1202_3173_amd import binding as sw

KERNEL, RECORD, WAIT, TAKE, POP, JOINED = 1, 2, 3, 4, 5, 6
WS_BASE = 4 << 40
NSTREAM = 3


def _rows_of(fp):
    """Start address (bytes) of every row of a footprint, and the row length in bytes."""
    addr, rows, cols, ld, count, stride = fp
    starts = (addr + 8 * (np.arange(count, dtype=np.int64)[:, None] * stride + np.arange(rows, dtype=np.int64)[None, :] * ld)).ravel()
    return starts, 8 * cols


def _exact_overlap(f, g):
    """Do two footprints share an element?  Row intervals of f against those of g."""
    sf, lf = _rows_of(f)
    sg, lg = _rows_of(g)
    sg = np.sort(sg)
    # for each row of f: the last row of g starting before its end must end after its start
    k = np.searchsorted(sg, sf + lf, side="left") - 1          # last g row with start < f row's end
    ok = k >= 0
    return bool(np.any(ok & (sg[np.maximum(k, 0)] + lg > sf)))


def check_record(log, ws_bytes):
    """-> (violations, stats).  violations: list of human-readable strings, empty when the record is safe."""
    log = [int(v) for v in log]
    violations = []
    vc = np.zeros((NSTREAM, NSTREAM), dtype=np.int64)    # vc[c][s]: kernels of stream s that precede c's next kernel
    events = {}                                          # (stream, slot) -> clock of `stream` when last recorded
    # all footprints submitted so far
    cap = 1024
    f_lo = np.empty(cap, np.int64); f_hi = np.empty(cap, np.int64); f_st = np.empty(cap, np.int64)
    f_ix = np.empty(cap, np.int64); f_wr = np.empty(cap, bool); f_id = np.empty(cap, np.int64)
    fps = []                                             # id -> (footprint tuple, kernel description)
    nf = 0
    stack = []                                           # live workspace buffers (offset, bytes)
    stats = dict(kernels=[0] * NSTREAM, waits=0, joined=0, max_tracked=0, takes=0)
    i = 0
    since_compact = 0
    while i < len(log):
        kind = log[i]
        if kind == KERNEL:
            c, kid, nr, nw = log[i + 1:i + 5]
            i += 5
            mine = []
            for j in range(nr + nw):
                mine.append((tuple(log[i:i + 6]), j >= nr))
                i += 6
            idx = vc[c][c] + 1
            stats["kernels"][c] += 1
            desc = f"kernel kind {kid}, number {idx} of stream {c}"
            for fp, is_write in mine:
                addr, rows, cols, ld, count, stride = fp
                lo = addr
                hi = addr + 8 * ((count - 1) * stride + (rows - 1) * ld + cols)
                # workspace discipline
                if WS_BASE <= lo < WS_BASE + max(ws_bytes, 1) or WS_BASE < hi <= WS_BASE + max(ws_bytes, 1):
                    off_lo, off_hi = lo - WS_BASE, hi - WS_BASE
                    if not any(o <= off_lo and off_hi <= o + b for o, b in _merged(stack)):
                        violations.append(f"{desc} touches workspace bytes [{off_lo}, {off_hi}) outside the live buffers")
                if nf:
                    m = (f_st[:nf] != c) & (f_ix[:nf] > vc[c][f_st[:nf]]) & (f_lo[:nf] < hi) & (lo < f_hi[:nf])
                    if not is_write:
                        m &= f_wr[:nf]
                    for k in np.nonzero(m)[0]:
                        other, odesc = fps[f_id[k]]
                        if _exact_overlap(fp, other):
                            violations.append(f"{desc} ({'writes' if is_write else 'reads'}) is not ordered after {odesc} "
                                              f"({'writes' if f_wr[k] else 'reads'}) on a common element")
                            if len(violations) > 20:
                                return violations, stats
            for fp, is_write in mine:
                if nf == cap:
                    cap *= 2
                    f_lo = np.resize(f_lo, cap); f_hi = np.resize(f_hi, cap); f_st = np.resize(f_st, cap)
                    f_ix = np.resize(f_ix, cap); f_wr = np.resize(f_wr, cap); f_id = np.resize(f_id, cap)
                addr, rows, cols, ld, count, stride = fp
                f_lo[nf] = addr
                f_hi[nf] = addr + 8 * ((count - 1) * stride + (rows - 1) * ld + cols)
                f_st[nf] = c; f_ix[nf] = idx; f_wr[nf] = is_write; f_id[nf] = len(fps)
                fps.append((fp, desc))
                nf += 1
            vc[c][c] = idx
            since_compact += 1
            if since_compact >= 256 and nf:
                # a kernel of stream s that every OTHER stream is already ordered after precedes all future kernels
                floor = np.array([min(vc[c2][s] for c2 in range(NSTREAM) if c2 != s) for s in range(NSTREAM)])
                keep = f_ix[:nf] > floor[f_st[:nf]]
                k = int(keep.sum())
                for arr in (f_lo, f_hi, f_st, f_ix, f_wr, f_id):
                    arr[:k] = arr[:nf][keep]
                nf = k
                since_compact = 0
        elif kind == RECORD:
            s, slot = log[i + 1:i + 3]
            events[(s, slot)] = vc[s].copy()
            i += 3
        elif kind == WAIT:
            c, s, slot = log[i + 1:i + 4]
            if (s, slot) in events:                      # waiting for an event never recorded is a no-op in HIP
                vc[c] = np.maximum(vc[c], events[(s, slot)])
            stats["waits"] += 1
            i += 4
        elif kind == TAKE:
            off, nbytes = log[i + 1:i + 3]
            if off < 0 or off + nbytes > ws_bytes:
                violations.append(f"buffer [{off}, {off + nbytes}) reaches beyond the workspace of {ws_bytes} bytes")
            for o, b in stack:
                if off < o + b and o < off + nbytes:
                    violations.append(f"buffer [{off}, {off + nbytes}) overlaps the live buffer [{o}, {o + b})")
            stack.append((off, nbytes))
            stats["takes"] += 1
            i += 3
        elif kind == POP:
            mark = log[i + 1]
            stack = [(o, b) for o, b in stack if o < mark]
            for o, b in stack:
                if o + b > mark:
                    violations.append(f"stack cut back to {mark} inside the live buffer [{o}, {o + b})")
            i += 2
        elif kind == JOINED:
            stats["joined"] += 1
            stats["max_tracked"] = max(stats["max_tracked"], log[i + 1])
            i += 2
        else:
            raise AssertionError(f"unknown record kind {kind} at word {i}")
    return violations, stats


def _merged(stack):
    """Adjacent live buffers as maximal runs (a kernel's bounding range may span T, S, Q taken back to back)."""
    out = []
    for o, b in sorted(stack):
        if out and out[-1][0] + out[-1][1] >= o:
            out[-1] = (out[-1][0], max(out[-1][1], o + b - out[-1][0]))
        else:
            out.append((o, b))
    return out


def _orders(levels):
    return ["".join("B" if (mask >> i) & 1 else "D" for i in range(levels)) for mask in range(1 << levels)]


def _trace(M, N, K, levels, order, ws_bytes, overlap=1, odd_mode=sw.SW_ODD_PAD, withhold=-1, lds=None):
    lda, ldb, ldc = lds or (K, N, N)
    return sw.sw_trace_gemm(M, N, K, lda, ldb, ldc, levels, order, ws_bytes, overlap, odd_mode, withhold)


# ---- the checker itself: it must object to records that ARE unsafe ----------------------------------------------

def _k(stream, reads, writes, kid=4):
    out = [KERNEL, stream, kid, len(reads), len(writes)]
    for a in list(reads) + list(writes):
        out += [a, 4, 4, 4, 1, 0]        # a 4 x 4 matrix at address a
    return out


def test_checker_flags_an_unordered_write_after_read_and_accepts_the_ordered_one():
    racy = _k(0, [1000], [5000]) + [RECORD, 0, 0] + _k(1, [9000], [1000])
    v, _ = check_record(racy, 0)
    assert len(v) == 1 and "not ordered" in v[0]
    safe = _k(0, [1000], [5000]) + [RECORD, 0, 0, WAIT, 1, 0, 0] + _k(1, [9000], [1000])
    assert check_record(safe, 0)[0] == []


def test_checker_takes_the_event_as_last_recorded_and_follows_chains():
    # the event is recorded BEFORE the conflicting kernel: waiting for it orders nothing
    early = [RECORD, 0, 0] + _k(0, [], [1000]) + [WAIT, 1, 0, 0] + _k(1, [1000], [2000])
    assert len(check_record(early, 0)[0]) == 1
    # a chain 0 -> 2 -> 1 orders stream 1 after stream 0's kernel
    chain = (_k(0, [], [1000]) + [RECORD, 0, 0, WAIT, 2, 0, 0] + _k(2, [], [7000]) + [RECORD, 2, 0, WAIT, 1, 2, 0] +
             _k(1, [1000], [2000]))
    assert check_record(chain, 0)[0] == []
    # a re-recorded slot stands for the LATER kernel, which is what a waiter then gets
    rerec = (_k(0, [], [1000]) + [RECORD, 0, 5] + _k(0, [], [3000]) + [RECORD, 0, 5, WAIT, 1, 0, 5] + _k(1, [1000, 3000], [2000]))
    assert check_record(rerec, 0)[0] == []
    # reads of one element on two streams are not a conflict
    assert check_record(_k(0, [1000], [5000]) + _k(1, [1000], [6000]), 0)[0] == []


def test_checker_compares_elements_not_bounding_boxes():
    # two interleaved quadrant views (same rows, disjoint column halves) of one matrix with pitch 8
    left = [KERNEL, 0, 4, 0, 1, 8000, 4, 4, 8, 1, 0]
    right = [KERNEL, 1, 4, 0, 1, 8000 + 32, 4, 4, 8, 1, 0]
    assert check_record(left + right, 0)[0] == []
    shifted = [KERNEL, 1, 4, 0, 1, 8000 + 24, 4, 4, 8, 1, 0]     # one column to the left: now they share a column
    assert len(check_record(left + shifted, 0)[0]) == 1


def test_checker_workspace_discipline():
    ok = [TAKE, 0, 512, TAKE, 512, 512, POP, 512, TAKE, 512, 256, POP, 0]
    assert check_record(ok, 1024)[0] == []
    assert check_record([TAKE, 0, 512, TAKE, 256, 512], 1024)[0]          # overlap
    assert check_record([TAKE, 0, 2048], 1024)[0]                          # beyond the end
    outside = [TAKE, 0, 128] + [KERNEL, 0, 4, 0, 1, WS_BASE + 256, 4, 4, 4, 1, 0]
    assert check_record(outside, 1024)[0]                                  # touches workspace nobody took


# ---- the library's records ------------------------------------------------------------------------------------------

N5, L5 = 94080, 5


@pytest.mark.parametrize("order", _orders(L5))
def test_every_order_of_five_levels_at_n_94080(order):
    """All 32 step orders at the largest configuration's shape, with the least workspace and with all the
    library can use (second set of leaf-side buffers, rich DFS steps)."""
    lean = sw.sw_plan_memory(N5, L5, order)
    rich = sw.sw_plan_workspace(N5, L5, order, 1 << 50)
    for ws in sorted({lean, (lean + rich) // 2 // 256 * 256, rich}):
        log = _trace(N5, N5, N5, L5, order, ws)
        v, st = check_record(log, ws)
        assert v == [], (order, ws, v[:3])
        if "D" in order:
            assert st["kernels"][1] > 0 and st["kernels"][2] > 0      # it did run on three streams
        else:
            assert st["kernels"][1] == 0 and st["kernels"][2] == 0    # one chain of kernels: one stream


def test_ring_wrap_and_the_fallback_are_reached():
    """More kernels per stream than the event ring has slots, and a run in which the tracker falls back to
    ordering everything: both paths must be part of what the tests above cover."""
    order = "DDDDD"
    ws = sw.sw_plan_memory(N5, L5, order)
    v, st = check_record(_trace(N5, N5, N5, L5, order, ws), ws)
    assert v == []
    assert min(st["kernels"]) > 256
    joined = 0
    for o in _orders(L5):
        for ws in (sw.sw_plan_memory(N5, L5, o), sw.sw_plan_workspace(N5, L5, o, 1 << 50)):
            log = _trace(N5, N5, N5, L5, o, ws)
            joined += int(np.count_nonzero(log == JOINED) > 0 and check_record(log, ws)[1]["joined"] > 0)
    print("orders with a fall-back:", joined)
    assert joined > 0


@pytest.mark.parametrize("shape,levels,odd", [
    ((23520, 23520, 23520), 5, sw.SW_ODD_PAD),      # configuration 4
    ((16384, 16384, 16384), 4, sw.SW_ODD_PAD),      # configuration 3
    ((30000, 20000, 25000), 4, sw.SW_ODD_PAD),      # rectangular
    ((1001, 1001, 1001), 3, sw.SW_ODD_PAD),         # padded copies
    ((1001, 777, 1300), 3, sw.SW_ODD_PAD),
    ((1001, 1001, 1001), 3, sw.SW_ODD_PEEL),        # peeled rows and columns
    ((94097, 94097, 94097), 5, sw.SW_ODD_PEEL),
    ((1001, 777, 1300), 2, sw.SW_ODD_PEEL),
    ((1001, 1001, 1001), 3, sw.SW_ODD_PEEL_LEVELS),   # peeled at every odd level
    ((94097, 94097, 94097), 5, sw.SW_ODD_PEEL_LEVELS),
    ((255, 255, 255), 4, sw.SW_ODD_PEEL_LEVELS),      # odd at every level
    ((1001, 777, 1300), 2, sw.SW_ODD_PEEL_LEVELS),
])
def test_other_shapes_padding_and_peeling(shape, levels, odd):
    M, N, K = shape
    sw.sw_set_odd_mode(odd)
    try:
        for order in _orders(levels):
            lean = sw.sw_plan_memory_rect(M, N, K, levels, order)
            for ws in (lean, 2 * lean + (1 << 20), 8 * lean + (64 << 20)):
                log = _trace(M, N, K, levels, order, ws, odd_mode=odd, lds=(K + 8, N + 24, N + 16))
                v, _ = check_record(log, ws)
                assert v == [], (shape, order, ws, v[:3])
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)


def test_fixed_caps_and_one_stream():
    ws = sw.sw_plan_workspace(4096, 3, "DDB", 1 << 40)
    for overlap in (0, 1, 64):
        log = _trace(4096, 4096, 4096, 3, "DDB", ws, overlap=overlap)
        v, st = check_record(log, ws)
        assert v == []
        if overlap == 0:
            assert st["kernels"][1] == st["kernels"][2] == 0 and st["waits"] == 0


def test_a_withheld_range_is_found():
    """Plant the mistake the checker exists for: one declared range is kept from the dependency tracker (as if an
    rng(...) were missing from an op(...)).  Not every range matters (many are ordered by another dependency of
    the same kernel), but the ones that carry an ordering must be found."""
    n, levels = 4096, 3
    for order in ("DDB", "DBB", "DDD", "BDB"):
        ws = sw.sw_plan_workspace(n, levels, order, 1 << 40)
        clean = _trace(n, n, n, levels, order, ws)
        assert check_record(clean, ws)[0] == []
        declared = 0
        i, log = 0, [int(x) for x in clean]
        while i < len(log):                               # ranges declared = footprints logged (one per declared range or fewer)
            if log[i] == KERNEL:
                declared += log[i + 3] + log[i + 4]
                i += 5 + 6 * (log[i + 3] + log[i + 4])
            else:
                i += {RECORD: 3, WAIT: 4, TAKE: 3, POP: 2, JOINED: 2}[log[i]]
        found = 0
        tried = 0
        for w in range(0, declared, max(1, declared // 120)):
            tried += 1
            v, _ = check_record(_trace(n, n, n, levels, order, ws, withhold=w), ws)
            found += bool(v)
        print(order, "withheld ranges found:", found, "of", tried)
        assert found >= tried // 5, (order, found, tried)


def test_withholding_the_leaf_product_output_is_always_found():
    """The write range of a leaf product whose result the caller's stream folds into C carries the ordering
    between the product stream and the caller's stream: without it the post-addition may start early."""
    n, levels, order = 2048, 2, "DB"
    ws = sw.sw_plan_memory(n, levels, order)
    log = [int(x) for x in _trace(n, n, n, levels, order, ws)]
    # number the declared ranges and find the write range of every product kernel (kind 7)
    i, declared, targets = 0, 0, []
    while i < len(log):
        if log[i] == KERNEL:
            nr, nw = log[i + 3], log[i + 4]
            if log[i + 2] == 7:
                targets.append(declared + nr)
            declared += nr + nw
            i += 5 + 6 * (nr + nw)
        else:
            i += {RECORD: 3, WAIT: 4, TAKE: 3, POP: 2, JOINED: 2}[log[i]]
    assert len(targets) == 7
    for w in targets:
        v, _ = check_record(_trace(n, n, n, levels, order, ws, withhold=w), ws)
        assert v, w
