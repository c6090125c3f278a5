"""Benchmark of the Strassen-Winograd fp64 product on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5]

A step is one whole product C = A*B (pre-additions, the BFS/DFS walk, batched leaf GEMMs, post-additions) on
inputs already resident in HBM.  The default workload is the fifth configuration (n = 94080, five levels,
step order chosen by the planner for the free device memory), the one the headline metric is quoted on:
effective GFLOP/s = 2 n^3 / t (Section 5.2).  One JSON line is printed, with
  roofline      the batched leaf GEMM (dominant kernel) against the fp64 matrix-core peak: actual flops
                2 m^3 per leaf product, per launch, over the average launch time measured with HIP events
                on the launch stream during the timed steps (where addition kernels run beside it on other
                streams and stretch its launches);
  single_stream one more product, outside the timed region, with everything on one stream: the same
                kernels' undisturbed rates (leaf GEMM against the MFMA peak, additions against HBM);
  cpu_baseline  the CPU oracle timed on this host on one leaf-sized classical product and scaled through
                the closed-form operation count (Appendix A) to the metric's unit.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP64_MFMA_PEAK_TFLOPS = 78.6     # MI355X dense fp64 matrix peak (published)
HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E peak (published)


def cpu_baseline(n, levels):
    """Oracle (as it stands, one thread) on one m x m classical leaf, m = n / 2^levels, scaled to the whole
    product through F(n) = c_s n^w0 - 5 n^2: effective GFLOP/s = 2 n^3 / (F(n) / rate)."""
    import importlib.util
    import numpy as np
    spec = importlib.util.spec_from_file_location("sw_oracle", os.path.join(ROOT, "oracle", "sw_oracle.py"))
    sw_oracle = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(sw_oracle)
    from paper_1202_3173_amd import binding, inputs
    m = n >> levels
    reps = 1
    while reps * 2.0 * m ** 3 < 1e11 and reps < 65536:     # about 100 GFLOP of CPU work: 10-20 s on one core
        reps *= 2
    A = inputs.matrix(m, 99, 0, "uniform")
    B = inputs.matrix(m, 99, 1, "uniform")
    t0 = time.perf_counter()
    for _ in range(reps):
        sw_oracle.gemm(A, B, 0)
    dt = time.perf_counter() - t0
    rate = reps * (2.0 * m ** 3 - m * m) / dt                # oracle's actual flop/s
    total = binding.sw_flop_count(n, levels)
    eff = 2.0 * n ** 3 / (total / rate) / 1e9
    return {"value": round(eff, 3), "unit": "GFLOP/s", "cores": 1, "kind": "oracle",
            "sample": f"{reps} classical {m}x{m}x{m} leaf product(s) of the {7 ** levels} ({dt:.1f} s, "
                      f"{rate / 1e9:.2f} actual GFLOP/s), scaled by the closed-form flop count F(n) of the "
                      f"{levels}-level product"}


def measured_traffic(m, batch):
    """HBM bytes per leaf-GEMM launch from the committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE
    runs, each scaled by a copy kernel of known size); None when no summary covers this launch shape."""
    path = os.path.join(ROOT, "profiles", f"leaf_gemm_m{m}_b{batch}_pmc.txt")
    key = f"leaf_gemm_m{m}_b{batch}_traffic_bytes_per_launch="
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line[len(key):])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg5", help="cfg1..cfg5 (default cfg5, the metric's configuration)")
    ap.add_argument("--schedule", default=None, help="override the step order: B/D characters, or `planner` for the planner's pick "
                                                        "(default: the configuration's, or the planner's where it names none)")
    ap.add_argument("--n", type=int, default=None, help="override the configuration's n (other sizes than the five)")
    ap.add_argument("--levels", type=int, default=None, help="override the number of levels (0 = the classical MFMA product)")
    ap.add_argument("--odd-mode", choices=["pad", "peel", "peel-levels"], default="pad",
                    help="when 2^levels does not divide n: zero-padded copies, one peel at the top, or a peel at every odd level")
    ap.add_argument("--overlap", type=int, default=None, help="0: one stream; 1 (default): three streams, leaf-side addition kernels sized to their work; k > 1: capped at k workgroups")
    ap.add_argument("--scheme", default="winograd",
                    help="the block scheme under the recursion (Section 6.6): winograd (default, the Strassen-Winograd path), strassen, "
                         "classical, laderman, classical3, or one per level separated by commas (top level first), e.g. "
                         "strassen,strassen,strassen,strassen,laderman")
    ap.add_argument("--budget-gb", type=float, default=None,
                    help="total device memory the product may use, in GB of 10^9 bytes, A, B and C included "
                         "(default: what is free on the device)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reference", action="store_true", help="skip the extra single-stream product after the timed steps")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1202_3173_amd import binding as sw
    from paper_1202_3173_amd import inputs

    cfg = dict(next(c for c in inputs.CONFIGS if c["name"] == args.config))
    if args.n is not None:
        cfg.update(n=args.n, name=f"{cfg['name']} with n={args.n}", schedule=None)
    if args.levels is not None:
        cfg.update(levels=args.levels, name=f"{cfg['name']} with levels={args.levels}", schedule=None)
    sw.sw_set_odd_mode({"pad": sw.SW_ODD_PAD, "peel": sw.SW_ODD_PEEL, "peel-levels": sw.SW_ODD_PEEL_LEVELS}[args.odd_mode])
    if args.overlap is not None:
        sw.sw_set_overlap(args.overlap)
    n, levels = cfg["n"], cfg["levels"]
    dev = "cuda:0"
    torch.cuda.set_device(0)

    A, B = inputs.device_pair(cfg, dev)
    C = torch.empty((n, n), dtype=torch.float64, device=dev)
    free, total_mem = torch.cuda.mem_get_info()
    budget = int(free - (2 << 30))
    if args.budget_gb is not None:
        budget = min(budget, int(args.budget_gb * 1e9) - 3 * n * n * 8)
        if budget < 0:
            sys.exit(f"bench.py: A, B and C alone take {3 * n * n * 8 / 1e9:.1f} GB")
    ids = {"winograd": sw.SW_SCHEME_WINOGRAD, "strassen": sw.SW_SCHEME_STRASSEN, "classical": sw.SW_SCHEME_CLASSICAL,
           "laderman": sw.SW_SCHEME_LADERMAN, "classical3": sw.SW_SCHEME_CLASSICAL3}
    names = args.scheme.split(",")
    if any(x not in ids for x in names) or (len(names) > 1 and "winograd" in names):
        sys.exit("bench.py: --scheme takes winograd, or strassen / classical / laderman / classical3 (one, or one per level)")
    per_level = [ids[x] for x in names] if len(names) > 1 else None
    scheme = ids[names[0]]
    if per_level is not None:
        levels = len(per_level)
        cfg.update(levels=levels, schedule=None)
    elif scheme != sw.SW_SCHEME_WINOGRAD:
        per_level = [scheme] * levels
    radix = 1
    for x in (per_level or [sw.SW_SCHEME_WINOGRAD] * levels):
        radix *= sw.SCHEME_BASE[x]
    if scheme == sw.SW_SCHEME_WINOGRAD:
        schedule = (None if args.schedule == "planner" else args.schedule or cfg["schedule"]) or sw.sw_plan_schedule(n, levels, budget)
        if levels == 0:
            schedule = ""
        need = sw.sw_plan_workspace(n, levels, schedule, budget)   # the minimum plus what the library can use
    else:
        # the comparison schemes: most BFS steps that fit, then least memory (the library's own preference)
        orders = ["".join("B" if (mask >> i) & 1 else "D" for i in range(levels)) for mask in range(1 << levels)]
        batch_of = lambda o: int(__import__("math").prod(sw.SCHEME_PRODUCTS[x] for x, ch in zip(per_level, o) if ch == "B"))
        fits = [(-o.count("B"), sw.sw_plan_memory_bilinear_levels(n, o, per_level), o) for o in orders]
        fits = [f for f in fits if f[1] <= budget and batch_of(f[2]) <= 4096]
        if args.schedule is None and not fits:
            sys.exit("bench.py: no step order of this scheme fits the free device memory")
        schedule = args.schedule if args.schedule is not None else min(fits)[2]
        need = sw.sw_plan_memory_bilinear_levels(n, schedule, per_level)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    if scheme != sw.SW_SCHEME_WINOGRAD:
        sw.sw_set_workspace(ws)
        sw.sw_set_stream(stream)

    def step():
        if scheme == sw.SW_SCHEME_WINOGRAD:
            sw.sw_gemm_ex(n, A, n, B, n, C, n, levels, schedule, ws, stream)
        else:
            sw.sw_gemm_bilinear_levels(n, A, B, C, schedule, per_level)

    def run_steps(count, what):
        """Enqueue `count` products back to back (no host synchronisation between the launches) and report each one on
        stderr when the GPU has finished it: an event per product on the launch stream, waited for by a reporter thread
        (the enqueueing thread itself is held back by the depth of the HIP queues and gets to the events late)."""
        import queue
        import threading
        done = queue.Queue()

        def report():
            k = 0
            while True:
                ev = done.get()
                if ev is None:
                    return
                ev.synchronize()
                k += 1
                print(f"bench.py: {what} product {k} of {count} done", file=sys.stderr, flush=True)

        t = threading.Thread(target=report, daemon=True)
        t.start()
        for _ in range(count):
            step()
            ev = torch.cuda.Event()
            ev.record()
            done.put(ev)
        done.put(None)
        torch.cuda.synchronize()
        t.join()

    run_steps(args.warmup, "warm-up")
    torch.cuda.synchronize()
    sw.sw_profile_enable(True)
    t0 = time.perf_counter()
    run_steps(args.steps, "timed")
    dt = time.perf_counter() - t0
    prof = sw.sw_profile_read()
    sw.sw_profile_enable(False)

    # The timed steps carry two HIP events around every kernel (that is where the roofline's launch durations come
    # from).  One more product without them, outside the timed region, shows what the brackets cost.
    plain_ms = None
    if not args.no_reference:
        t2 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        plain_ms = (time.perf_counter() - t2) * 1e3

    # The timed steps run with the library's default executor (three streams: additions beside the leaf
    # products), where the leaf kernel shares the machine with the addition kernels and its launches stretch.
    # One more product on a single stream (not part of `value`) gives the same kernel's undisturbed rate.
    alone = None
    if scheme == sw.SW_SCHEME_WINOGRAD and levels > 0 and args.overlap != 0 and not args.no_reference:
        sw.sw_set_overlap(0)
        sw.sw_profile_enable(True)
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        dt1 = time.perf_counter() - t1
        p1 = sw.sw_profile_read()
        sw.sw_profile_enable(False)
        sw.sw_set_overlap(1 if args.overlap is None else args.overlap)
        l1 = p1["leaf_gemm"]
        a_bytes = sum(p1[k]["work"] for k in ("pre_add", "post_add", "dfs_add", "pad"))
        a_ms = sum(p1[k]["ms"] for k in ("pre_add", "post_add", "dfs_add", "pad"))
        alone = {"ms_per_step": round(dt1 * 1e3, 3), "effective_GFLOPs": round(2.0 * n ** 3 / dt1 / 1e9, 1),
                 "leaf_TFLOPs": round(l1["work"] / (l1["ms"] * 1e-3) / 1e12, 3) if l1["ms"] > 0 else 0.0,
                 "leaf_frac_of_peak": round(l1["work"] / (l1["ms"] * 1e-3) / 1e12 / FP64_MFMA_PEAK_TFLOPS, 4) if l1["ms"] > 0 else 0.0,
                 "leaf_avg_launch_ms": round(l1["ms"] / max(1, l1["launches"]), 4),
                 "additions_GBps": round(a_bytes / (a_ms * 1e-3) / 1e9, 1) if a_ms > 0 else 0.0,
                 "additions_frac_of_hbm_peak": round(a_bytes / (a_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if a_ms > 0 else 0.0}

    ms_per_step = dt * 1e3 / args.steps
    eff_gflops = 2.0 * n ** 3 / (dt / args.steps) / 1e9

    leaf = prof["leaf_gemm"]
    leaf_batch = 1                                                                  # leaves per launch
    for x, ch in zip(per_level or [sw.SW_SCHEME_WINOGRAD] * levels, schedule):
        leaf_batch *= sw.SCHEME_PRODUCTS[x] if ch == "B" else 1
    leaf_tflops = leaf["work"] / (leaf["ms"] * 1e-3) / 1e12 if leaf["ms"] > 0 else 0.0
    roofline = {"bound": "mfma", "kernel": "leaf_gemm_kernel (batched fp64 MFMA)",
                "achieved": round(leaf_tflops, 3), "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(leaf_tflops / FP64_MFMA_PEAK_TFLOPS, 4),
                "traffic": measured_traffic(n // radix, leaf_batch),
                "traffic_source": "the committed rocprofv3 counter summary of this launch shape under profiles/ (FETCH_SIZE and WRITE_SIZE "
                                  "runs scaled by a copy of known size); a constant, not measured in this run; null when no summary covers the shape",
                "launches": leaf["launches"], "avg_launch_ms": round(leaf["ms"] / max(1, leaf["launches"]), 4),
                "flops_per_launch": leaf["work"] / max(1, leaf["launches"]),
                "note": ("timed with the default executor: addition kernels run beside the leaf launches on other streams and "
                         "stretch them; `single_stream` has the same kernel undisturbed" if alone else None)}
    adds = {}
    add_bytes = add_ms = 0.0
    if prof["peel"]["launches"]:
        adds["peel_products"] = {"TFLOPs": round(prof["peel"]["work"] / (prof["peel"]["ms"] * 1e-3) / 1e12, 2),
                                 "ms_per_step": round(prof["peel"]["ms"] / args.steps, 3)}
    for k in ("pre_add", "post_add", "dfs_add", "pad"):
        p = prof[k]
        if p["launches"]:
            adds[k] = {"GBps": round(p["work"] / (p["ms"] * 1e-3) / 1e9, 1), "ms_per_step": round(p["ms"] / args.steps, 3),
                       "launches_per_step": p["launches"] // args.steps}
            add_bytes += p["work"]
            add_ms += p["ms"]
    add_gbps = add_bytes / (add_ms * 1e-3) / 1e9 if add_ms > 0 else 0.0

    # cheap end-to-end sanity on the timed result (Freivalds, one +-1 vector, torch's own GEMV)
    g = torch.Generator(device="cpu").manual_seed(1)
    x = (torch.randint(0, 2, (n,), generator=g, dtype=torch.int64) * 2 - 1).to(torch.float64).to(dev)
    check = float((torch.mv(C, x) - torch.mv(A, torch.mv(B, x))).abs().max())
    absmax = lambda t: max(float(t[r:r + 4096].abs().max()) for r in range(0, n, 4096))   # chunked: no n x n temporary
    tol = 1e-10 * n * absmax(A) * absmax(B)

    # the algorithm's own operation count (closed form; one scheme for all levels, n divisible by the levels' radices)
    flops_actual = sw.sw_flop_count_bilinear(n, levels, scheme) if (n % radix == 0 and len(names) == 1) else None

    out = {
        "metric": "effective fp64 GFLOP/s (2n^3/t)", "value": round(eff_gflops, 1), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: n={n} square fp64 C=A*B, {levels} "
                               + ({"winograd": "Strassen-Winograd", "strassen": "Strassen (original)", "classical": "recursive classical",
                                   "laderman": "Laderman (3 x 3 blocks)", "classical3": "recursive classical (3 x 3 blocks)"}[names[0]]
                                  if len(names) == 1 else "mixed (" + args.scheme + ")") + " levels, "
                               f"leaf {-(-n // radix)}, entries {cfg['dist']} seed {cfg['seed']}"
                               + (f", odd size handled by {args.odd_mode if scheme == sw.SW_SCHEME_WINOGRAD else 'pad'}" if n % radix else ""),
                   "n": n, "levels": levels, "schedule": schedule, "workspace_GB": round(need / 1e9, 3),
                   "hbm_total_GB": round(total_mem / 1e9, 1),
                   "memory_budget_GB": args.budget_gb, "operands_plus_workspace_GB": round((3 * n * n * 8 + need) / 1e9, 3)},
        "pct_of_fp64_mfma_peak": round(100.0 * eff_gflops / (FP64_MFMA_PEAK_TFLOPS * 1e3), 2),
        "actual_flops_per_step": flops_actual,
        # Section 6.3's yardstick: the time the algorithm's own flop count would take at the machine's peak
        "pct_of_algorithm_peak": (round(100.0 * flops_actual / (dt / args.steps) / (FP64_MFMA_PEAK_TFLOPS * 1e12), 2)
                                  if flops_actual else None),
        "roofline": roofline,
        "additions": {"GBps_all": round(add_gbps, 1), "frac_of_hbm_peak": round(add_gbps / HBM_PEAK_GBPS, 4),
                      "ms_per_step": round(add_ms / args.steps, 3), "by_class": adds,
                      "note": ("kernel time summed over streams: the leaf-side addition kernels run capped at 32 workgroups "
                               "beside the products, so their own rate is low by design; `single_stream` has them alone" if alone else None)},
        "leaf_ms_per_step": round(leaf["ms"] / args.steps, 3),
        "event_brackets": {"in_timed_region": True, "kernels_per_step": sum(p["launches"] for p in prof.values()) // max(1, args.steps),
                           "one_product_without_them_ms": None if plain_ms is None else round(plain_ms, 3),
                           "note": "every kernel of the timed steps is bracketed by two HIP events on its launch stream (the source of "
                                   "roofline.avg_launch_ms); one more product without the brackets is timed after the timed region"},
        "single_stream": alone,
        "check": {"freivalds_max_abs_diff": check, "tolerance": tol, "ok": check <= tol},
        "paper_context": "Cray XT4: 49.1 effective GFLOPS/node, 33% above the classical peak (Section 5.2)",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(n, levels)     # always the Strassen-Winograd oracle
    print(json.dumps(out))
    if check > tol:
        sys.exit(1)


if __name__ == "__main__":
    main()
