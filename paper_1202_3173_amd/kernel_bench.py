"""Time the single steps of the path through the C ABI, each against the roofline that bounds it.

  python -m paper_1202_3173_amd.kernel_bench leaf --m 2940 --batch 49        # fp64 MFMA peak
  python -m paper_1202_3173_amd.kernel_bench pre_add --h 2940 --live 7       # HBM bandwidth
  python -m paper_1202_3173_amd.kernel_bench post_add --h 2940 --live 7      # HBM bandwidth
  python -m paper_1202_3173_amd.kernel_bench copy --bytes 8589934592         # torch's device copy, for scale
  python -m paper_1202_3173_amd.kernel_bench dgemm --M 60000 --N 40000 --K 50000 --transa 1 --levels -1
                                                                            # the general product (alpha, beta,
                                                                            # transposes, rectangular), 2MNK/t

  python -m paper_1202_3173_amd.kernel_bench depth --sizes 4096,8192 --max-levels 6
                                                                            # whole product against the depth,
                                                                            # next to what sw_plan_levels picks
  python -m paper_1202_3173_amd.kernel_bench orders --n 16384 --levels 4     # whole product for every step order
                                                                            # that fits, next to the planner's pick
  python -m paper_1202_3173_amd.kernel_bench streams --bytes 8589934592       # synthetic kernels with r input and w
                                                                            # output streams: what HBM sustains
  python -m paper_1202_3173_amd.kernel_bench beside --m 2940 --batch 49       # leaf products next to background
                                                                            # traffic, with the shader clock
  python -m paper_1202_3173_amd.kernel_bench mfma                             # the fp64 matrix pipes on registers alone
  python -m paper_1202_3173_amd.kernel_bench error_growth --n 2048           # error against the depth, with and
                                                                            # without diagonal scaling (Section 6.1)

Each kernel is launched `--iters` times between two HIP events on the launch stream; one JSON line reports
the average duration and the achieved rate on ALGORITHMIC work: 2 m^3 flops per leaf product; for the
additions the distinct elements read plus written, times 8 bytes (pre-add: 4 quadrants in, 7 operands out;
post-add: 7 products in, 4 quadrants out).  The same commands run under rocprofv3 give the summaries kept
under profiles/.
"""
import argparse
import json
import sys

FP64_MFMA_PEAK_TFLOPS = 78.6
HBM_PEAK_GBPS = 8000.0


def _timed(fn, iters, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()                 # the binding launches on torch's current stream, which these events share
    for _ in range(iters):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def _best_of(fn, reps=3):
    """Wall time of the best of `reps` runs after one warm-up (whole products: host-side clock around a sync)."""
    import time
    import torch
    best = float("inf")
    for rep in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        if rep:
            best = min(best, time.perf_counter() - t0)
    return best


def depth_study(sizes, max_levels):
    """For every n and every depth the planner's step order for the free device memory is timed on seeded uniform
    inputs generated in HBM; one line per (n, depth) and one per n with the measured optimum and the model's choice."""
    import torch
    from . import binding as sw
    from . import inputs
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    for n in sizes:
        A, B = inputs.device_pair({"n": n, "seed": 11, "dist": "uniform"}, dev)
        C = torch.empty((n, n), dtype=torch.float64, device=dev)
        free, _ = torch.cuda.mem_get_info()
        budget = int(free - (2 << 30))
        rows = []
        for L in range(0, max_levels + 1):
            if (n >> L) < 64:
                break
            try:
                order = sw.sw_plan_schedule(n, L, budget) if L else ""
            except sw.SwError:
                continue
            ws = torch.empty(max(sw.sw_plan_workspace(n, L, order, budget), 256), dtype=torch.uint8, device=dev)
            best = _best_of(lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, L, order, ws, stream))
            del ws
            rows.append((L, order, best))
            print(f"n {n} levels {L} order {order or '-'} ms {best * 1e3:.3f} effective_TFLOPs {2.0 * n ** 3 / best / 1e12:.2f}", flush=True)
        measured = min(rows, key=lambda r: r[2])
        picked = sw.sw_plan_levels(n, budget)
        t_picked = next(r[2] for r in rows if r[0] == picked)
        print(f"n {n}: measured optimum {measured[0]} levels ({measured[2] * 1e3:.3f} ms), sw_plan_levels picks {picked} "
              f"({t_picked * 1e3:.3f} ms, {100.0 * (t_picked / measured[2] - 1):.1f} % above the optimum)", flush=True)
        del A, B, C
        torch.cuda.empty_cache()


def order_study(n, levels, dist, seed):
    """Every step order of `levels` steps that fits the free device memory, timed on the whole product, next to the
    planner's pick (sw_plan_schedule) for the same budget."""
    import torch
    from . import binding as sw
    from . import inputs
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    A, B = inputs.device_pair({"n": n, "seed": seed, "dist": dist}, dev)
    C = torch.empty((n, n), dtype=torch.float64, device=dev)
    free, _ = torch.cuda.mem_get_info()
    budget = int(free - (2 << 30))
    picked = sw.sw_plan_schedule(n, levels, budget)
    rows = []
    for mask in range(1 << levels):
        order = "".join("B" if (mask >> i) & 1 else "D" for i in range(levels))
        if sw.sw_plan_memory(n, levels, order) > budget:
            continue
        ws = torch.empty(max(sw.sw_plan_workspace(n, levels, order, budget), 256), dtype=torch.uint8, device=dev)
        t = _best_of(lambda: sw.sw_gemm_ex(n, A, n, B, n, C, n, levels, order, ws, stream))
        del ws
        torch.cuda.empty_cache()
        rows.append((order, t))
        print(f"n {n} order {order} ms {t * 1e3:.3f} effective_TFLOPs {2.0 * n ** 3 / t / 1e12:.2f}" + ("   <- planner" if order == picked else ""), flush=True)
    best = min(rows, key=lambda r: r[1])
    t_picked = next(t for o, t in rows if o == picked)
    print(f"n {n} levels {levels}: best order {best[0]} ({best[1] * 1e3:.3f} ms), planner picks {picked} ({t_picked * 1e3:.3f} ms, "
          f"{100.0 * (t_picked / best[1] - 1):.1f} % above the best)", flush=True)


def stream_sweep(total_bytes, iters):
    """The rate of one-pass streaming kernels against the number of streams read and written at once (16-byte
    accesses, non-temporal, full grid), as a markdown table: bytes moved = (inputs + outputs) x stream length."""
    import ctypes
    import os
    import torch
    L = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsw_probe.so"))
    L.sw_probe_streams.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream().cuda_stream
    print("| streams in | streams out | pieces per workgroup and stream | GB per launch | ms | TB/s | of 8 TB/s |")
    print("|---|---|---|---|---|---|---|")
    shapes = [(0, 1), (1, 0), (1, 1), (2, 1), (4, 1), (1, 4), (1, 8), (4, 4), (8, 8), (16, 16), (5, 3), (4, 7), (7, 4), (16, 49), (49, 16)]
    cases = [(i, o, 1) for i, o in shapes] + [(i, o, 4) for i, o in [(1, 8), (4, 7), (7, 4), (16, 49)]]
    for nin, nout, chunks in cases:
        n2 = total_bytes // (nin + nout) // 16
        n2 -= n2 % 4096
        stride = n2 + 4096 + 16            # streams a little more than their length apart, never a power of two
        a = torch.rand(max(nin, 1) * stride * 2, dtype=torch.float64, device=dev)
        o = torch.empty(max(nout, 1) * stride * 2, dtype=torch.float64, device=dev)
        blocks = min((n2 + 256 * chunks - 1) // (256 * chunks), 1 << 20)

        def launch():
            rc = L.sw_probe_streams(nin, nout, chunks, a.data_ptr(), o.data_ptr(), n2, stride, stride, blocks, st)
            assert rc == 0, rc
        ms = _timed(launch, iters, 2)
        moved = (nin + nout) * n2 * 16
        rate = moved / (ms * 1e-3) / 1e12
        print(f"| {nin} | {nout} | {chunks} | {moved / 1e9:.2f} | {ms:.3f} | {rate:.2f} | {100 * rate / 8.0:.0f} % |", flush=True)
        del a, o
        torch.cuda.empty_cache()


def beside_study(m, batch, launches):
    """The leaf products next to background traffic: `launches` launches of `batch` products of m^3 on one stream while a
    streaming kernel of a chosen number of workgroups runs on another and a one-wavefront meter reads the shader
    clock on a third.  Markdown table: background, its rate, the median launch, its rate, the average shader clock."""
    import ctypes
    import os
    import time
    import torch
    from . import binding as sw
    X = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsw_probe.so"))
    X.sw_probe_load.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    X.sw_probe_meter.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    s_gemm, s_load, s_meter = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    n2 = (2 << 30) // 16
    src = torch.rand(n2 * 2, dtype=torch.float64, device=dev)
    dst = torch.empty(n2 * 2, dtype=torch.float64, device=dev)
    stamps = torch.zeros(4, dtype=torch.int64, device=dev)
    ld = (m + 15) // 16 * 16
    if ld >= 256 and ld % 256 == 0:
        ld += 16
    stride = (ld * m + 31) // 32 * 32
    A = torch.rand(batch * stride, dtype=torch.float64, device=dev) - 0.5
    B = torch.rand(batch * stride, dtype=torch.float64, device=dev) - 0.5
    C = torch.empty(batch * stride, dtype=torch.float64, device=dev)
    flops = 2.0 * m ** 3 * batch
    print(f"| background beside {batch} products of {m}^3 | its rate while the products run, TB/s | median launch ms | TFLOP/s | of the fp64 MFMA peak | shader clock MHz |")
    print("|---|---|---|---|---|---|")
    for label, mode, blocks in [("none", 0, 0), ("copy, 32 workgroups", 0, 32), ("copy, 96 workgroups", 0, 96), ("copy, 256 workgroups", 0, 256),
                                ("read only, 96 workgroups", 1, 96), ("write only, 96 workgroups", 2, 96), ("none", 0, 0)]:
        torch.cuda.synchronize()
        # the meter runs for about three quarters of the time the launches take (about 3.5 us per iteration), so it
        # ends while they still run; the background traffic is cut into pieces of a few milliseconds, timed one by one,
        # enough of them to outlast the products
        est_ms = launches * flops / 50e12 * 1e3
        assert X.sw_probe_meter(stamps.data_ptr(), int(0.75 * launches * flops / 75e12 * 1e6 / 3.5), s_meter.cuda_stream) == 0
        pieces = []
        if blocks:
            reps = max(1, blocks // 32)
            for _ in range(int(est_ms / 2.0) + 8):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(s_load)
                assert X.sw_probe_load(src.data_ptr(), dst.data_ptr(), n2, reps, mode, blocks, s_load.cuda_stream) == 0
                e1.record(s_load)
                pieces.append((e0, e1))
            time.sleep(0.01)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
        ev[0].record(s_gemm)
        for i in range(launches):
            with torch.cuda.stream(s_gemm):
                sw.sw_leaf_gemm(m, batch, A, ld, stride, B, ld, stride, C, ld, stride)
            ev[i + 1].record(s_gemm)
        torch.cuda.synchronize()
        t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(1, launches))
        mid = t[len(t) // 2]
        st = stamps.cpu().tolist()
        mhz = (st[1] - st[0]) / ((st[3] - st[2]) / 100.0)
        rate = "-"
        if blocks:
            # pieces that ran wholly while the products ran: those that began after the first launch ended and ended
            # before the last launch did
            inside = [p for p in pieces if ev[1].elapsed_time(p[0]) > 0 and p[1].elapsed_time(ev[launches]) > 0]
            if inside:
                span = inside[0][0].elapsed_time(inside[-1][1])
                moved = len(inside) * reps * n2 * 16 * (2 if mode == 0 else 1)
                rate = f"{moved / span / 1e9:.2f}"
        print(f"| {label} | {rate} | {mid:.3f} | {flops / mid / 1e9:.1f} | {flops / mid / 1e9 / FP64_MFMA_PEAK_TFLOPS:.3f} | {mhz:.0f} |", flush=True)


def mfma_peak(iters):
    """What the fp64 matrix pipes sustain without any memory traffic: 512 workgroups (two per CU) of four wavefronts,
    each issuing rounds of 16 independent v_mfma_f64_16x16x4_f64 on registers; the shader clock is read beside it."""
    import ctypes
    import os
    import torch
    X = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsw_probe.so"))
    X.sw_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    X.sw_probe_meter.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    blocks, rounds = 512, 200000
    out = torch.empty(blocks * 256, dtype=torch.float64, device=dev)
    stamps = torch.zeros(4, dtype=torch.int64, device=dev)
    s_meter = torch.cuda.Stream()
    st = torch.cuda.current_stream().cuda_stream
    flops = blocks * 4 * rounds * 16 * 2048.0

    def launch():
        assert X.sw_probe_mfma(out.data_ptr(), blocks, rounds, st) == 0
    _timed(launch, 2, 1)                                          # bring the clock up
    expect_ms = flops / 75e12 * 1e3
    assert X.sw_probe_meter(stamps.data_ptr(), int(0.75 * iters * expect_ms * 1e3 / 3.5), s_meter.cuda_stream) == 0
    ms = _timed(launch, iters, 0)
    torch.cuda.synchronize()
    t = stamps.cpu().tolist()
    mhz = (t[1] - t[0]) / ((t[3] - t[2]) / 100.0)
    rate = flops / (ms * 1e-3) / 1e12
    print(json.dumps({"kernel": "mfma_f64_16x16x4 on registers", "workgroups": blocks, "avg_ms": round(ms, 3), "TFLOPs": round(rate, 2),
                      "frac_of_fp64_mfma_peak": round(rate / FP64_MFMA_PEAK_TFLOPS, 4), "shader_clock_MHz": round(mhz),
                      "TFLOPs_at_2400_MHz": round(rate * 2400.0 / mhz, 2)}))


def error_growth(n):
    """Markdown tables: the largest entry-wise error relative to ||A(i,:)|| ||B(:,j)|| (the quantity the scaled bound
    of Section 6.1 is stated in) in units of n*eps, and in brackets the norm-wise error in units of
    n*eps*||A||*||B|| (max-norms), against a product accumulated in extended precision on the host."""
    import numpy as np
    import torch
    from . import binding as sw
    from . import inputs
    dev = "cuda:0"

    def run(A, B, levels, mode):
        dA, dB = torch.from_numpy(A).to(dev), torch.from_numpy(B).to(dev)
        C = torch.empty((n, n), dtype=torch.float64, device=dev)
        schedule = "B" * levels
        ws = torch.empty(sw.sw_plan_memory_scaled(n, levels, schedule), dtype=torch.uint8, device=dev)
        sw.sw_set_workspace(ws)
        sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
        try:
            sw.sw_gemm_scaled(n, dA, dB, C, levels, schedule, mode)
            torch.cuda.synchronize()
        finally:
            sw.sw_set_workspace(None)
            sw.sw_set_stream(0)
        return C.cpu().numpy()

    eps = np.finfo(float).eps
    for dist in ("badscaled", "rowscaled", "uniform"):
        A = inputs.matrix(n, 77, 0, dist)
        B = inputs.matrix(n, 77, 1, dist)
        ref = (A.astype(np.longdouble) @ B.astype(np.longdouble)).astype(np.float64)
        rowcol = np.max(np.abs(A), axis=1)[:, None] * np.max(np.abs(B), axis=0)[None, :]
        norm = np.max(np.abs(A)) * np.max(np.abs(B))
        print(f"\n### {dist}, n = {n}\n")
        print("| levels | plain | outside (D1, D3) | inside (D2) | both |")
        print("|---|---|---|---|---|")
        for levels in range(0, 6):
            cells = []
            for mode in (0, sw.SW_SCALE_OUTSIDE, sw.SW_SCALE_INSIDE, sw.SW_SCALE_OUTSIDE | sw.SW_SCALE_INSIDE):
                C = run(A, B, levels, mode)
                cells.append(f"{np.max(np.abs(C - ref) / rowcol) / (n * eps):.3g} [{np.max(np.abs(C - ref)) / (n * eps * norm):.2g}]")
            print(f"| {levels} | " + " | ".join(cells) + " |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("kernel", choices=["leaf", "pre_add", "post_add", "pre_add2", "post_add2", "copy", "dgemm", "depth", "orders", "streams", "beside", "mfma", "error_growth"])
    ap.add_argument("--sizes", default="2048,4096,8192,16384,23520,32768,47040", help="depth: the sizes n")
    ap.add_argument("--max-levels", type=int, default=6, help="depth: the largest depth tried")
    ap.add_argument("--n", type=int, default=2048, help="orders, error_growth: the size n")
    ap.add_argument("--dist", default="uniform", help="orders: input distribution")
    ap.add_argument("--seed", type=int, default=11)
    ap.add_argument("--M", type=int, default=40000)
    ap.add_argument("--N", type=int, default=40000)
    ap.add_argument("--K", type=int, default=40000)
    ap.add_argument("--transa", type=int, default=0)
    ap.add_argument("--transb", type=int, default=0)
    ap.add_argument("--levels", type=int, default=-1, help="dgemm: recursion depth, -1 = the library's cost model")
    ap.add_argument("--alpha", type=float, default=1.0)
    ap.add_argument("--beta", type=float, default=0.0)
    ap.add_argument("--m", type=int, default=2940)
    ap.add_argument("--batch", type=int, default=49)
    ap.add_argument("--h", type=int, default=2940)
    ap.add_argument("--live", type=int, default=7)
    ap.add_argument("--side", type=int, default=0)
    ap.add_argument("--bytes", type=int, default=8 << 30)
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    args = ap.parse_args()
    if args.kernel == "depth":
        return depth_study([int(x) for x in args.sizes.split(",")], args.max_levels)
    if args.kernel == "orders":
        if args.levels < 1:
            sys.exit("kernel_bench orders: give --levels (1 or more)")
        return order_study(args.n, args.levels, args.dist, args.seed)
    if args.kernel == "error_growth":
        return error_growth(args.n)
    if args.kernel == "streams":
        return stream_sweep(args.bytes, args.iters)
    if args.kernel == "beside":
        return beside_study(args.m, args.batch, args.iters)
    if args.kernel == "mfma":
        return mfma_peak(args.iters)

    import torch
    from paper_1202_3173_amd import binding as sw
    dev = "cuda:0"
    torch.cuda.set_device(0)
    # same workspace layout rule as the library: pitch a multiple of 16 doubles, never of 256
    def pitch(h):
        ld = (h + 15) // 16 * 16
        return ld + 16 if ld >= 256 and ld % 256 == 0 else ld

    if args.kernel == "leaf":
        m, b = args.m, args.batch
        ld = pitch(m)
        stride = (ld * m + 31) // 32 * 32
        A = torch.rand(b * stride, dtype=torch.float64, device=dev) - 0.5
        B = torch.rand(b * stride, dtype=torch.float64, device=dev) - 0.5
        C = torch.empty(b * stride, dtype=torch.float64, device=dev)
        ms = _timed(lambda: sw.sw_leaf_gemm(m, b, A, ld, stride, B, ld, stride, C, ld, stride), args.iters, args.warmup)
        flops = 2.0 * m ** 3 * b
        rate = flops / (ms * 1e-3) / 1e12
        out = {"kernel": "leaf_gemm", "m": m, "batch": b, "ld": ld, "avg_ms": round(ms, 4), "TFLOPs": round(rate, 2),
               "frac_of_fp64_mfma_peak": round(rate / FP64_MFMA_PEAK_TFLOPS, 4)}
    elif args.kernel == "dgemm":
        M, N, K = args.M, args.N, args.K
        shape_a = (K, M) if args.transa else (M, K)
        shape_b = (N, K) if args.transb else (K, N)
        A = torch.rand(shape_a, dtype=torch.float64, device=dev) - 0.5
        B = torch.rand(shape_b, dtype=torch.float64, device=dev) - 0.5
        C = torch.rand((M, N), dtype=torch.float64, device=dev)
        free, _ = torch.cuda.mem_get_info()
        ws = torch.empty(int(free - (3 << 30)), dtype=torch.uint8, device=dev)
        sw.sw_set_workspace(ws)
        sw.sw_set_stream(torch.cuda.current_stream().cuda_stream)
        ms = _timed(lambda: sw.sw_dgemm(args.transa, args.transb, M, N, K, args.alpha, A, shape_a[1], B, shape_b[1],
                                        args.beta, C, N, args.levels, None), args.iters, args.warmup)
        sw.sw_set_workspace(None)
        eff = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        out = {"kernel": "sw_dgemm", "M": M, "N": N, "K": K, "transa": args.transa, "transb": args.transb,
               "levels": args.levels if args.levels >= 0 else "auto (block shape and depth by the library's cost model)",
               "avg_ms": round(ms, 3), "achieved": round(eff, 2), "unit": "effective TFLOP/s (2MNK/t)",
               "peak": FP64_MFMA_PEAK_TFLOPS, "frac": round(eff / FP64_MFMA_PEAK_TFLOPS, 4), "bound": "mfma"}
    elif args.kernel in ("pre_add2", "post_add2"):
        m, live = args.h, args.live                 # --h is the grandchild size here: the parent is 4 m x 4 m
        n = 4 * m
        ld = pitch(m)
        cs = (ld * m + 31) // 32 * 32
        pld = pitch(n)
        ps = (pld * n + 31) // 32 * 32
        P = torch.rand(live * ps, dtype=torch.float64, device=dev)
        K = torch.rand(live * 49 * cs, dtype=torch.float64, device=dev)
        if args.kernel == "pre_add2":
            ms = _timed(lambda: sw.sw_pre_add2(args.side, P, pld, ps, live, m, K, ld, cs), args.iters, args.warmup)
        else:
            ms = _timed(lambda: sw.sw_post_add2(K, ld, cs, live, m, P, pld, ps), args.iters, args.warmup)
        nbytes = 8.0 * live * m * m * 65
        rate = nbytes / (ms * 1e-3) / 1e9
        out = {"kernel": args.kernel, "m": m, "live": live, "avg_ms": round(ms, 4), "GBps": round(rate, 1),
               "frac_of_hbm_peak": round(rate / HBM_PEAK_GBPS, 4)}
    elif args.kernel in ("pre_add", "post_add"):
        h, live = args.h, args.live
        n = 2 * h
        ld = pitch(h)
        cs = (ld * h + 31) // 32 * 32
        pld = pitch(n)
        ps = (pld * n + 31) // 32 * 32
        P = torch.rand(live * ps, dtype=torch.float64, device=dev)
        K = torch.rand(live * 7 * cs, dtype=torch.float64, device=dev)
        if args.kernel == "pre_add":
            ms = _timed(lambda: sw.sw_pre_add(args.side, P, pld, ps, live, h, K, ld, cs), args.iters, args.warmup)
        else:
            ms = _timed(lambda: sw.sw_post_add(K, ld, cs, live, h, P, pld, ps), args.iters, args.warmup)
        nbytes = 8.0 * live * h * h * 11
        rate = nbytes / (ms * 1e-3) / 1e9
        out = {"kernel": args.kernel, "h": h, "live": live, "avg_ms": round(ms, 4), "GBps": round(rate, 1),
               "frac_of_hbm_peak": round(rate / HBM_PEAK_GBPS, 4)}
    else:
        nb = args.bytes
        s = torch.empty(nb, dtype=torch.uint8, device=dev)
        d = torch.empty(nb, dtype=torch.uint8, device=dev)
        s.zero_()
        ms = _timed(lambda: d.copy_(s), args.iters, args.warmup)
        rate = 2.0 * nb / (ms * 1e-3) / 1e9
        out = {"kernel": "torch_copy", "bytes": nb, "avg_ms": round(ms, 4), "GBps_read_plus_write": round(rate, 1),
               "frac_of_hbm_peak": round(rate / HBM_PEAK_GBPS, 4)}
    print(json.dumps(out))


if __name__ == "__main__":
    sys.exit(main())
