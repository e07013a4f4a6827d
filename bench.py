#!/usr/bin/env python3
"""Benchmark of the binned exact kNN hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--n-bins N] [--d-bin D]

A step is one pass of the whole hot path over one batch of synthetic input already resident
in HBM: bounding box + bin assignment + counting sort (fg_bin_points), the exact
shell-expanding query on that binning (fg_query_binned; the two together are what
fg_binned_select_knn runs) and, when the configuration has a backward pass, the backward
scatter in the same bin order (fg_knn_backward_binned: a training step bins its points once).  The headline workload is configuration 3: 1,000,000
points, d = 3, 10 row splits, K = 32.  One JSON line is printed on stdout.

Besides the contract fields the line carries
  roofline      the query kernel against the HBM roofline: algorithmic bytes per launch
                (per query: K*(4+4) output + d*4 coordinates + 4 permutation entry, plus the
                bin-boundary table once) over the kernel's mean duration, measured live with
                events on the launch stream
  cpu_baseline  the CPU oracle as it stands, timed on this machine's host cores on a bounded
                sample of the same workload (a reported baseline, not a target)
  stages        mean milliseconds of binning / query / backward and candidate evaluations/s
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak


def _traffic_from_profiles(name: str):
    """Measured HBM bytes per launch of the query kernel, if a summary was committed."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--n-bins", type=int, default=0)
    ap.add_argument("--d-bin", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=100000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (segments are independent and would "
              "shard across GPUs with no exchange, but nothing here uses a second GPU); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2511_10442_amd import binding as B
    from paper_2511_10442_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = W.CONFIGS[args.config]()
    n, d, k, s = w.n, w.d, w.k, w.n_segments
    x = torch.from_numpy(w.coords).to(dev)
    rs = torch.from_numpy(w.row_splits).to(dev)
    g = torch.from_numpy(w.grad_d2).to(dev) if w.backward else None
    ws_bytes = max(B.fg_workspace_size(n, d, s, k, args.n_bins, args.d_bin), B.fg_workspace_size(n, d, s, k))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)   # forward bins as asked, backward bins automatically
    out_idx = torch.empty((n, k), dtype=torch.int32, device=dev)
    out_d2 = torch.empty((n, k), dtype=torch.float32, device=dev)
    grad = torch.empty((n, d), dtype=torch.float32, device=dev) if w.backward else None

    def step():
        binning = B.fg_bin_points(x, rs, k, args.n_bins, args.d_bin, ws)
        B.fg_query_binned(binning, rs, k, out_idx, out_d2)
        if w.backward:
            B.fg_knn_backward_binned(binning, g, out_idx, x, grad)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = n * args.steps / (t1 - t0)

    # ---- per-stage timing with events on the launch stream (torch's current stream)
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

    reps = max(5, args.steps)
    binning = B.fg_bin_points(x, rs, k, args.n_bins, args.d_bin, ws)
    ms_bin = timed(lambda: B.fg_bin_points(x, rs, k, args.n_bins, args.d_bin, ws), reps)
    binning = B.fg_bin_points(x, rs, k, args.n_bins, args.d_bin, ws)
    ms_query = timed(lambda: B.fg_query_binned(binning, rs, k, out_idx, out_d2), reps)
    deferred = int(binning.work_count.item())                     # of the timed query launches
    cand = torch.empty((n,), dtype=torch.int32, device=dev)
    B.fg_query_binned(binning, rs, k, out_idx, out_d2, cand)      # counting instantiation, never timed
    torch.cuda.synchronize()
    total_cand = int(cand.to(torch.int64).sum().item())
    ms_bwd = timed(lambda: B.fg_knn_backward_binned(binning, g, out_idx, x, grad), reps) if w.backward else None
    # the stand-alone backward bins once more, into the same workspace: `binning` is dead from here on
    ms_bwd_alone = timed(lambda: B.fg_knn_backward(g, out_idx, x, rs, grad, ws), reps) if w.backward else None

    total_bins = binning.n_segments * binning.cells_per_segment
    algo_bytes = n * (k * 8 + d * 4 + 4) + (total_bins + 1) * 4
    achieved = algo_bytes / (ms_query * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "query stage = k_query_tile_sorted (dominant) + k_query_list_wave + the tile-order kernels",
                "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": _traffic_from_profiles("query_kernel_%s_traffic.txt" % w.name.split("_")[0]),
                "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": round(ms_query, 4)}

    # the same stage against what actually bounds it: one float32 operation per lane and clock (no FMA by the
    # definition of the distance, packed float32 off): 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
    alu_peak = 256 * 4 * 16 * 2.4e9 / 1e12
    alu_achieved = total_cand * (3 * d - 1) / (ms_query * 1e-3) / 1e12
    roofline_alu = {"bound": "alu", "achieved": round(alu_achieved, 3), "peak": round(alu_peak, 1), "unit": "TFLOP/s",
                    "frac": round(alu_achieved / alu_peak, 5),
                    "note": "distance arithmetic only (3d-1 float32 operations per candidate); selection work not counted"}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        rows = np.random.Generator(np.random.PCG64(7)).choice(n, size=min(args.cpu_rows, n), replace=False)
        rows = np.sort(rows).astype(np.int64)
        c0 = time.perf_counter()
        oracle.knn_rows(w.coords, w.row_splits, k, rows)
        c1 = time.perf_counter()
        cpu = {"value": round(len(rows) / (c1 - c0), 1), "unit": "queries/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "%d random query rows of %s, each against its full row split (forward only), %.1f s wall"
                         % (len(rows), w.name, c1 - c0)}

    line = {
        "metric": "kNN queries/sec + achieved HBM GB/s (% peak), 1M pts d=3 k=32",
        "value": round(value, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.note, "name": w.name, "n": n, "d": d, "k": k, "segments": s,
                   "n_bins": binning.n_bins, "d_bin": binning.d_bin,
                   "step": "fg_bin_points + fg_query_binned" + (" + fg_knn_backward_binned" if w.backward else "")},
        "roofline": roofline,
        "roofline_alu": roofline_alu,
        "cpu_baseline": cpu,
        "stages": {"binning_ms": round(ms_bin, 4), "query_ms": round(ms_query, 4),
                   "backward_ms": None if ms_bwd is None else round(ms_bwd, 4),
                   "backward_standalone_ms": None if ms_bwd_alone is None else round(ms_bwd_alone, 4),
                   "query_only_queries_per_s": round(n / (ms_query * 1e-3), 1),
                   "candidates_per_query": round(total_cand / n, 2),
                   "queries_handed_to_list_kernel": deferred,
                   "candidate_evals_per_s": round(total_cand / (ms_query * 1e-3), 1),
                   "hbm_frac_of_peak_query": round(achieved / HBM_PEAK_GBS, 5)},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
