"""Measured time of the Strassen-Winograd product against the recursion depth, next to what sw_plan_levels picks.

  python -m paper_1202_3173_amd.depth_study [--sizes 4096,8192,...] [--max-levels 6]

For every n and every depth the planner's step order for the free device memory is timed (best of three
after one warm-up) on seeded uniform inputs generated in HBM; one line per (n, depth) and one per n with the
measured optimum and the model's choice.
"""
import argparse
import time

import torch

from . import binding as sw
from . import inputs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", default="2048,4096,8192,16384,23520,32768,47040")
    ap.add_argument("--max-levels", type=int, default=6)
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    for n in [int(x) for x in args.sizes.split(",")]:
        cfg = {"n": n, "seed": 11, "dist": "uniform"}
        A, B = inputs.device_pair(cfg, dev)
        C = torch.empty((n, n), dtype=torch.float64, device=dev)
        free, _ = torch.cuda.mem_get_info()
        budget = int(free - (2 << 30))
        rows = []
        for L in range(0, args.max_levels + 1):
            if (n >> L) < 64:
                break
            try:
                order = sw.sw_plan_schedule(n, L, budget) if L else ""
            except sw.SwError:
                continue
            need = sw.sw_plan_workspace(n, L, order, budget)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
            best = float("inf")
            for rep in range(4):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                sw.sw_gemm_ex(n, A, n, B, n, C, n, L, order, ws, stream)
                torch.cuda.synchronize()
                if rep:
                    best = min(best, time.perf_counter() - t0)
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


if __name__ == "__main__":
    main()
