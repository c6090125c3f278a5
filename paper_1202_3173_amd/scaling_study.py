"""Error growth of the product with the number of Strassen-Winograd levels, with and without the diagonal
scaling of Section 6.1, on the GPU, for three input distributions.

  python -m paper_1202_3173_amd.scaling_study [--n 2048]

Prints markdown tables: the largest entry-wise error relative to ||A(i,:)|| ||B(:,j)|| (the quantity the
scaled bound of Section 6.1 is stated in) in units of n*eps, and in brackets the norm-wise error in units of
n*eps*||A||*||B|| (max-norms), against a product accumulated in extended precision on the host.
"""
import argparse

import numpy as np


def run(sw, torch, A, B, levels, mode):
    n = A.shape[0]
    dev = "cuda:0"
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=2048)
    args = ap.parse_args()
    import torch
    from paper_1202_3173_amd import binding as sw
    from paper_1202_3173_amd import inputs
    n = args.n
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
                C = run(sw, torch, A, B, levels, mode)
                cells.append(f"{np.max(np.abs(C - ref) / rowcol) / (n * eps):.3g} [{np.max(np.abs(C - ref)) / (n * eps * norm):.2g}]")
            print(f"| {levels} | " + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()
