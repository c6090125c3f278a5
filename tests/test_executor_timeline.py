"""How well the executor's three streams can overlap, estimated on the host.

The record of `sw_trace_gemm` (every kernel with the memory it touches, every event record and stream wait) is replayed
with a duration for each kernel -- leaf products at 70 TFLOP/s, everything else at 5.2 TB/s on the elements it reads and
writes -- and the semantics of HIP streams: a stream runs its kernels in order, a wait holds the waiting stream's later
kernels until the kernel before the event's record has finished.  The replay knows nothing of interference between
kernels that run at the same time, so its times are lower bounds; what it does show is every moment the leaf-product
stream stands still because of a DEPENDENCY (operands not formed yet, a buffer still in use), which is what the second
set of leaf-side buffers, the order of the additions and the early thin products of the peeled levels are there to
avoid.  A change that serialises the streams again fails here, without a GPU.
"""
import numpy as np
import pytest

from paper_1202_3173_amd import binding as sw

KERNEL, RECORD, WAIT, TAKE, POP, JOINED = 1, 2, 3, 4, 5, 6
K_GEMM = 7
NSTREAM = 3
S_MM = 2                       # the stream of the leaf products (0: the caller's, post-additions; 1: pre-additions)
LEAF_RATE, HBM_RATE = 70e12, 5.2e12


def replay(log):
    """-> dict(makespan, leaf_busy, leaf_stream, by_stream): seconds."""
    log = [int(v) for v in log]
    t = [0.0] * NSTREAM              # when each stream's last kernel finishes
    hold = [0.0] * NSTREAM           # earliest start of the stream's next kernel because of waits
    events = {}
    busy = [0.0] * NSTREAM
    leaf = 0.0
    i = 0
    while i < len(log):
        kind = log[i]
        if kind == KERNEL:
            c, kid, nr, nw = log[i + 1:i + 5]
            i += 5
            fps = [tuple(log[i + 6 * j:i + 6 * j + 6]) for j in range(nr + nw)]
            i += 6 * (nr + nw)
            elems = sum(rows * cols * count for (_, rows, cols, _, count, _) in fps)
            dur = 8.0 * elems / HBM_RATE
            if kid == K_GEMM:
                (_, m, k, _, count, _), (_, _, n, _, _, _) = fps[0], fps[1]
                if min(m, n, k) >= 64:                       # a real product, not a one-wide strip
                    dur = 2.0 * m * n * k * count / LEAF_RATE
                    leaf += dur
            start = max(t[c], hold[c])
            t[c] = start + dur
            busy[c] += dur
        elif kind == RECORD:
            s, slot = log[i + 1:i + 3]
            events[(s, slot)] = t[s]
            i += 3
        elif kind == WAIT:
            c, s, slot = log[i + 1:i + 4]
            if (s, slot) in events:
                hold[c] = max(hold[c], events[(s, slot)])
            i += 4
        elif kind in (TAKE,):
            i += 3
        elif kind in (POP, JOINED):
            if kind == JOINED:                               # every stream was ordered after every other
                top = max(t)
                hold = [max(h, top) for h in hold]
            i += 2
        else:
            raise AssertionError(f"unknown record kind {kind} at word {i}")
    return dict(makespan=max(t), leaf_busy=leaf, by_stream=busy)


def _run(n, levels, order, ws, odd_mode=sw.SW_ODD_PAD, overlap=1):
    return replay(sw.sw_trace_gemm(n, n, n, n, n, n, levels, order, ws, overlap, odd_mode, -1))


# ---- the replay itself -----------------------------------------------------------------------------------------------

def _k(stream, kid, fps_r, fps_w):
    out = [KERNEL, stream, kid, len(fps_r), len(fps_w)]
    for f in list(fps_r) + list(fps_w):
        out += list(f)
    return out


def test_replay_orders_streams_only_through_waits():
    a = (1000, 1000, 1000, 1000, 1, 0)                       # 10^6 elements: 8 MB, 1.54 us at 5.2 TB/s
    one = 8e6 / HBM_RATE
    free = replay(_k(0, 4, [a], []) + _k(1, 4, [a], []))
    assert free["makespan"] == pytest.approx(one)            # nothing orders them: side by side
    chained = replay(_k(0, 4, [a], []) + [RECORD, 0, 0, WAIT, 1, 0, 0] + _k(1, 4, [a], []))
    assert chained["makespan"] == pytest.approx(2 * one)
    early = replay([RECORD, 0, 0] + _k(0, 4, [a], []) + [WAIT, 1, 0, 0] + _k(1, 4, [a], []))
    assert early["makespan"] == pytest.approx(one)           # the event was recorded before the kernel
    g = replay(_k(2, K_GEMM, [(0, 128, 256, 256, 3, 0), (0, 256, 512, 512, 3, 0)], [(0, 128, 512, 512, 3, 0)]))
    assert g["leaf_busy"] == pytest.approx(2.0 * 128 * 512 * 256 * 3 / LEAF_RATE)


# ---- the library's records -------------------------------------------------------------------------------------------

def test_headline_configuration_keeps_the_leaf_stream_busy():
    """n = 94080, five levels, the planner's order with the workspace the library can use of 93 GB: once the first
    operands are formed the leaf products never wait for an addition; what is exposed is the start and the end."""
    n, levels = 94080, 5
    budget = 93 * 10 ** 9
    order = sw.sw_plan_schedule(n, levels, budget)
    assert order == "DDDBB"
    ws = sw.sw_plan_workspace(n, levels, order, budget)
    r = _run(n, levels, order, ws)
    assert r["leaf_busy"] == pytest.approx(7 ** 5 * 2.0 * 2940 ** 3 / LEAF_RATE)
    assert r["leaf_busy"] / r["makespan"] > 0.97
    # with the least workspace there is one set of leaf-side buffers: additions and products take turns
    lean = _run(n, levels, order, sw.sw_plan_memory(n, levels, order))
    assert lean["makespan"] > r["makespan"] * 1.05
    assert lean["leaf_busy"] == pytest.approx(r["leaf_busy"])
    # one stream: the sum of everything
    single = _run(n, levels, order, ws, overlap=0)
    assert single["makespan"] == pytest.approx(sum(single["by_stream"]))
    assert single["makespan"] > r["makespan"] * 1.08


@pytest.mark.parametrize("n,levels", [(23520, 5), (16384, 4), (47040, 4)])
def test_planner_orders_of_other_sizes_overlap(n, levels):
    budget = 290 * 10 ** 9 - 3 * n * n * 8
    order = sw.sw_plan_schedule(n, levels, budget)
    ws = sw.sw_plan_workspace(n, levels, order, budget)
    r = _run(n, levels, order, ws)
    single = _run(n, levels, order, ws, overlap=0)
    if "D" in order:
        assert r["leaf_busy"] / r["makespan"] > 0.90, (order, r)
        assert r["makespan"] < 0.95 * single["makespan"]
    else:
        assert r["makespan"] == pytest.approx(single["makespan"])


def test_peeling_at_every_level_does_not_stall_the_leaf_stream():
    """n = 94097 peeled level by level (the odd level 5881 lies between the two BFS steps): the one-wide products that
    read the operands run before the step, so the next problem's operands are formed while this one's leaf
    products run.  With them after the step the leaf stream stood still for a fifth of the time."""
    n, levels = 94097, 5
    sw.sw_set_odd_mode(sw.SW_ODD_PEEL_LEVELS)
    try:
        budget = 93 * 10 ** 9
        order = sw.sw_plan_schedule(n, levels, budget)
        ws = sw.sw_plan_workspace(n, levels, order, budget)
        r = _run(n, levels, order, ws, odd_mode=sw.SW_ODD_PEEL_LEVELS)
    finally:
        sw.sw_set_odd_mode(sw.SW_ODD_PAD)
    assert order == "DDDBB"
    assert r["leaf_busy"] / r["makespan"] > 0.95, r
