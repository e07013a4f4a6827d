"""The paper's own benchmark shape, this library's side only (Section 4: uniformly distributed
random vectors, 1e3 .. 5e6 points, dimension sweep at N = 1M and K = 40, size sweeps at d = 3 and
d = 5, K in {10, 40, 100}; the comparison libraries of the paper are not part of this build).

    python -m paper_2511_10442_amd.sweep_uniform [--quick] [--out profiles/uniform_sweep.md]

For every point of the sweep: forward time (binning + query, mean of `reps` runs after one
warm-up, events on the launch stream), queries/s, candidates per query, and the time of the
same call with n_bins = 1 (every query scans its whole row split through the same kernels:
this library's own brute force), which is where the binned search stops paying off as d grows.
A sample of rows of every run is checked against the CPU oracle unless --no-check is given.
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="fewer and smaller points")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--out", default="")
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2511_10442_amd import binding as B
    from paper_2511_10442_amd import workloads as W

    dev = "cuda:0"

    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    points = []
    big = 200_000 if args.quick else 1_000_000
    for d in range(2, 11):                                   # dimension sweep (Fig. 1 shape)
        points.append(("dim", big, d, 40))
    sizes = [1000, 10_000, 100_000] + ([] if args.quick else [1_000_000, 5_000_000])
    for d in (3, 5):                                         # size sweeps (Figs. 2 and 3 shape)
        for n in sizes:
            points.append(("size d=%d" % d, n, d, 40))
    for k in (10, 100):                                      # neighbour-count sweep at d = 3
        for n in sizes:
            points.append(("k=%d" % k, n, 3, k))

    lines = ["| sweep | N | d | K | n_bins x d_bin | forward ms | queries/s | candidates/query | brute force ms (n_bins=1) | speed-up | checked rows |",
             "|---|---|---|---|---|---|---|---|---|---|---|"]
    for name, n, d, k in points:
        x_np, rs_np = W.uniform(n, d, seed=4000 + d)
        x = torch.from_numpy(x_np).to(dev)
        rs = torch.from_numpy(rs_np).to(dev)
        ws = B.alloc_workspace(n, d, 1, k, 0, 0, dev)
        oi = torch.empty((n, k), dtype=torch.int32, device=dev)
        od = torch.empty((n, k), dtype=torch.float32, device=dev)
        ms = timed(lambda: B.fg_binned_select_knn(x, rs, k, 0, 0, ws, oi, od), args.reps)
        _, _, cand = B.fg_binned_select_knn_counted(x, rs, k, 0, 0, ws)
        torch.cuda.synchronize()
        cpq = float(cand.to(torch.float64).mean().item())
        nb, db = B.fg_auto_n_bins(n, 1, k, d, 1)
        brute = ""
        speed = ""
        if n * n <= 1.1e12 / max(1, d // 3):                 # keep the brute-force leg bounded
            ws1 = B.alloc_workspace(n, d, 1, k, 1, 2, dev)
            msb = timed(lambda: B.fg_binned_select_knn(x, rs, k, 1, 2, ws1, oi, od), 1 if n >= 1_000_000 else 2)
            brute, speed = "%.3f" % msb, "%.1f" % (msb / ms)
            B.fg_binned_select_knn(x, rs, k, 0, 0, ws, oi, od)
        checked = 0
        if not args.no_check:
            import oracle
            rows = np.sort(np.random.Generator(np.random.PCG64(9)).choice(n, size=min(n, 200), replace=False)).astype(np.int64)
            ri, rd = oracle.knn_rows(x_np, rs_np, k, rows)
            torch.cuda.synchronize()
            gi, gd = oi.cpu().numpy()[rows], od.cpu().numpy()[rows]
            assert np.array_equal(gi, ri) and np.array_equal(gd.view(np.uint32), rd.view(np.uint32)), (name, n, d, k)
            checked = len(rows)
        line = "| %s | %d | %d | %d | %d x %d | %.3f | %.3g | %.1f | %s | %s | %d |" % (
            name, n, d, k, nb, db, ms, n / (ms * 1e-3), cpq, brute, speed, checked)
        print(line, flush=True)
        lines.append(line)
        del ws
    if args.out:
        with open(args.out, "w") as f:
            f.write("Uniform random vectors, forward only, one MI355X; command: python -m paper_2511_10442_amd.sweep_uniform"
                    + (" --quick" if args.quick else "") + "\n\n" + "\n".join(lines) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
