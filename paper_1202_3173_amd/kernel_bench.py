"""Time the single steps of the path through the C ABI, each against the roofline that bounds it.

  python -m paper_1202_3173_amd.kernel_bench leaf --m 2940 --batch 49        # fp64 MFMA peak
  python -m paper_1202_3173_amd.kernel_bench pre_add --h 2940 --live 7       # HBM bandwidth
  python -m paper_1202_3173_amd.kernel_bench post_add --h 2940 --live 7      # HBM bandwidth
  python -m paper_1202_3173_amd.kernel_bench copy --bytes 8589934592         # torch's device copy, for scale
  python -m paper_1202_3173_amd.kernel_bench dgemm --M 60000 --N 40000 --K 50000 --transa 1 --levels -1
                                                                            # the general product (alpha, beta,
                                                                            # transposes, rectangular), 2MNK/t

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("kernel", choices=["leaf", "pre_add", "post_add", "copy", "dgemm"])
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
