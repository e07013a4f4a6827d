#!/usr/bin/env python3
"""Benchmark of the binned exact kNN hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--n-bins N] [--d-bin D] [--all-configs]
    python bench.py --sweep uniform [--quick] [--out profiles/uniform_sweep.md]
    python bench.py --profile-stage query|forward|backward|step|oc|none [--config C] [--reps R] [--calib-mb M]

Default mode.  A step is one pass of the whole hot path over one batch of synthetic input already resident
in HBM: bounding box + bin assignment + counting sort (fg_bin_points), the exact shell-expanding query on
that binning (fg_query_binned; the two together are what fg_binned_select_knn runs) and, when the
configuration has a backward pass, the backward scatter in the same bin order (fg_knn_backward_binned: a
training step bins its points once).  The headline workload is configuration 3: 1,000,000 points, d = 3,
10 row splits, K = 32.  One JSON line is printed on stdout.  Besides the contract fields it carries
  roofline      the query stage against the HBM roofline: algorithmic bytes per launch (per query:
                K*(4+4) output + d*4 coordinates + 4 permutation entry, plus the bin-boundary table once)
                over the stage's mean duration, measured live with events on the launch stream; also as a
                fraction of the copy bandwidth measured in the same run (a plain device-to-device copy)
  roofline_alu  the same stage against the float32 issue rate (what actually bounds it)
  cpu_baseline  the CPU oracle as it stands, timed on this machine's host cores on a bounded sample of the same
                workload, all cores and one core (a reported baseline, not a target)
  stages        mean milliseconds of binning / query / backward and candidate evaluations/s
  configs       with --all-configs: the same stage figures for all five configurations

--sweep uniform: the paper's own benchmark shape (Section 4: uniformly distributed random vectors, 1e3 .. 5e6
points, dimension sweep at N = 1M and K = 40, size sweeps at d = 3 and d = 5, K in {10, 40, 100}), this
library's side only; prints a markdown table with, per point, the time of the same call at n_bins = 1 (every
query scans its whole row split through the same kernels: this library's own brute force).  A sample of
rows of every run is checked against the CPU oracle unless --no-check is given.

--profile-stage: runs one stage a few times and exits, for rocprofv3 (kernel trace or counters);
--calib-mb M adds a plain elementwise copy over M MiB as the known-size reference for memory counters.
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
METRIC = "kNN queries/sec + achieved HBM GB/s (% peak), 1M pts d=3 k=32"


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


def _timed(torch, fn, reps):
    """Mean milliseconds of fn over reps calls, events on torch's current stream (the launch stream)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _copy_bandwidth(torch, dev):
    """GB/s (read + write) of a plain device-to-device copy of 1 GiB: what this chip's memory system sustains."""
    a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    b = torch.empty_like(a)
    ms = _timed(torch, lambda: b.copy_(a), 10)
    return 2.0 * a.numel() * 4 / (ms * 1e-3) / 1e9


class _Workload:
    """A configuration resident in HBM with its outputs and workspace."""

    def __init__(self, torch, B, w, dev, n_bins=0, d_bin=0):
        self.torch, self.B, self.w = torch, B, w
        self.n_bins, self.d_bin = n_bins, d_bin
        n, d, k, s = w.n, w.d, w.k, w.n_segments
        self.x = torch.from_numpy(w.coords).to(dev)
        self.rs = torch.from_numpy(w.row_splits).to(dev)
        self.g = torch.from_numpy(w.grad_d2).to(dev) if w.backward else None
        ws_bytes = max(B.fg_workspace_size(n, d, s, k, n_bins, d_bin), B.fg_workspace_size(n, d, s, k))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)   # forward bins as asked, backward bins automatically
        self.out_idx = torch.empty((n, k), dtype=torch.int32, device=dev)
        self.out_d2 = torch.empty((n, k), dtype=torch.float32, device=dev)
        self.grad = torch.empty((n, d), dtype=torch.float32, device=dev) if w.backward else None
        self.cand = torch.empty((n,), dtype=torch.int32, device=dev)

    def bin(self):
        return self.B.fg_bin_points(self.x, self.rs, self.w.k, self.n_bins, self.d_bin, self.ws)

    def step(self):
        binning = self.bin()
        self.B.fg_query_binned(binning, self.rs, self.w.k, self.out_idx, self.out_d2)
        if self.w.backward:
            self.B.fg_knn_backward_binned(binning, self.g, self.out_idx, self.x, self.grad)

    def stages(self, reps):
        """Per-stage mean times and counts."""
        torch, B, w = self.torch, self.B, self.w
        n, d, k = w.n, w.d, w.k
        ms_bin = _timed(torch, self.bin, reps)
        binning = self.bin()
        ms_query = _timed(torch, lambda: B.fg_query_binned(binning, self.rs, k, self.out_idx, self.out_d2), reps)
        deferred = int(binning.work_count.item())                     # of the timed query launches
        B.fg_query_binned(binning, self.rs, k, self.out_idx, self.out_d2, self.cand)      # counting instantiation, never timed
        torch.cuda.synchronize()
        total_cand = int(self.cand.to(torch.int64).sum().item())
        ms_bwd = ms_bwd_alone = None
        if w.backward:
            ms_bwd = _timed(torch, lambda: B.fg_knn_backward_binned(binning, self.g, self.out_idx, self.x, self.grad), reps)
            # the stand-alone backward bins once more, into the same workspace: `binning` is dead from here on
            ms_bwd_alone = _timed(torch, lambda: B.fg_knn_backward(self.g, self.out_idx, self.x, self.rs, self.grad, self.ws), reps)
        total_bins = binning.n_segments * binning.cells_per_segment
        algo_bytes = n * (k * 8 + d * 4 + 4) + (total_bins + 1) * 4
        bwd_bytes = 2 * n * k * 4 + 2 * n * d * 4
        return {"n_bins": binning.n_bins, "d_bin": binning.d_bin, "total_bins": total_bins,
                "binning_ms": ms_bin, "query_ms": ms_query, "backward_ms": ms_bwd, "backward_standalone_ms": ms_bwd_alone,
                "candidates": total_cand, "deferred": deferred, "query_bytes": algo_bytes, "backward_bytes": bwd_bytes}


def _stage_record(w, st):
    """Rounded, self-describing per-configuration record for the JSON line."""
    n, d = w.n, w.d
    q = st["query_ms"] * 1e-3
    rec = {"n": n, "d": d, "k": w.k, "segments": w.n_segments, "n_bins": st["n_bins"], "d_bin": st["d_bin"],
           "binning_ms": round(st["binning_ms"], 4), "query_ms": round(st["query_ms"], 4),
           "backward_ms": None if st["backward_ms"] is None else round(st["backward_ms"], 4),
           "backward_standalone_ms": None if st["backward_standalone_ms"] is None else round(st["backward_standalone_ms"], 4),
           "query_only_queries_per_s": round(n / q, 1),
           "candidates_per_query": round(st["candidates"] / n, 2),
           "queries_handed_to_list_kernel": st["deferred"],
           "candidate_evals_per_s": round(st["candidates"] / q, 1),
           "query_algorithmic_gbs": round(st["query_bytes"] / q / 1e9, 2),
           "hbm_frac_of_peak_query": round(st["query_bytes"] / q / 1e9 / HBM_PEAK_GBS, 5)}
    if st["backward_ms"] is not None:
        rec["backward_algorithmic_gbs"] = round(st["backward_bytes"] / (st["backward_ms"] * 1e-3) / 1e9, 2)
    return rec


def run_headline(args) -> int:
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
    wl = _Workload(torch, B, w, dev, args.n_bins, args.d_bin)

    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = n * args.steps / (t1 - t0)

    reps = max(5, args.steps)
    st = wl.stages(reps)
    copy_gbs = _copy_bandwidth(torch, dev)
    ms_query = st["query_ms"]
    achieved = st["query_bytes"] / (ms_query * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "query stage = k_query_tile_sorted (dominant) + k_query_list_wave + the tile-order kernels",
                "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": _traffic_from_profiles("query_kernel_%s_traffic.txt" % w.name.split("_")[0]),
                "algorithmic_bytes_per_launch": st["query_bytes"], "kernel_ms": round(ms_query, 4),
                "measured_copy_gbs": round(copy_gbs, 1), "frac_of_measured_copy": round(achieved / copy_gbs, 5)}

    # the same stage against what actually bounds it: one float32 operation per lane and clock (no FMA by the
    # definition of the distance, packed float32 off): 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
    alu_peak = 256 * 4 * 16 * 2.4e9 / 1e12
    alu_achieved = st["candidates"] * (3 * d - 1) / (ms_query * 1e-3) / 1e12
    roofline_alu = {"bound": "alu", "achieved": round(alu_achieved, 3), "peak": round(alu_peak, 1), "unit": "TFLOP/s",
                    "frac": round(alu_achieved / alu_peak, 5),
                    "note": "distance arithmetic only (3d-1 float32 operations per candidate); selection work not counted"}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.Generator(np.random.PCG64(7))
        rows = np.sort(rng.choice(n, size=min(args.cpu_rows, n), replace=False)).astype(np.int64)
        cores = oracle.num_threads()          # before the one-thread leg below changes the setting
        c0 = time.perf_counter()
        oracle.knn_rows(w.coords, w.row_splits, k, rows)
        c1 = time.perf_counter()
        rows1 = np.sort(rng.choice(n, size=min(2000, n), replace=False)).astype(np.int64)
        s0 = time.perf_counter()
        oracle.knn_rows(w.coords, w.row_splits, k, rows1, 1)
        s1 = time.perf_counter()
        seg_size = n / s
        cpu = {"value": round(len(rows) / (c1 - c0), 1), "unit": "queries/s", "cores": cores,
               "kind": "oracle",
               "sample": "%d random query rows of %s, each against its full row split (forward only), %.1f s wall"
                         % (len(rows), w.name, c1 - c0),
               "single_thread": {"value": round(len(rows1) / (s1 - s0), 1), "unit": "queries/s", "cores": 1,
                                 "pair_evals_per_s": round(len(rows1) * seg_size / (s1 - s0), 1),
                                 "sample": "%d random query rows, %.1f s wall" % (len(rows1), s1 - s0)}}

    line = {
        "metric": METRIC,
        "value": round(value, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.note, "name": w.name, "n": n, "d": d, "k": k, "segments": s,
                   "n_bins": st["n_bins"], "d_bin": st["d_bin"],
                   "step": "fg_bin_points + fg_query_binned" + (" + fg_knn_backward_binned" if w.backward else "")},
        "roofline": roofline,
        "roofline_alu": roofline_alu,
        "cpu_baseline": cpu,
        "stages": {key: val for key, val in _stage_record(w, st).items() if key not in ("n", "d", "k", "segments", "n_bins", "d_bin")},
    }
    if args.all_configs:
        del wl
        torch.cuda.empty_cache()
        table = {}
        for cfg in (1, 2, 3, 4, 5):
            wc = W.CONFIGS[cfg]()
            wlc = _Workload(torch, B, wc, dev)
            for _ in range(2):
                wlc.step()
            torch.cuda.synchronize()
            table[wc.name] = _stage_record(wc, wlc.stages(5))
            del wlc
            torch.cuda.empty_cache()
        line["configs"] = table
        if args.out:
            with open(args.out, "w") as f:
                f.write("Stage times of the five configurations, one MI355X, automatic bins; command: python bench.py --all-configs --out %s\n\n" % args.out)
                f.write("| config | N | d | K | splits | n_bins x d_bin | binning ms | query ms | backward ms | backward alone ms | candidates/query | handed to list kernel | query GB/s (algorithmic) | % of HBM peak |\n")
                f.write("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
                for name, r in table.items():
                    f.write("| %s | %d | %d | %d | %d | %d x %d | %.3f | %.3f | %s | %s | %.1f | %d | %.1f | %.2f |\n" % (
                        name, r["n"], r["d"], r["k"], r["segments"], r["n_bins"], r["d_bin"], r["binning_ms"], r["query_ms"],
                        "" if r["backward_ms"] is None else "%.3f" % r["backward_ms"],
                        "" if r["backward_standalone_ms"] is None else "%.3f" % r["backward_standalone_ms"],
                        r["candidates_per_query"], r["queries_handed_to_list_kernel"], r["query_algorithmic_gbs"],
                        100 * r["hbm_frac_of_peak_query"]))
    print(json.dumps(line))
    return 0


def run_sweep(args) -> int:
    import numpy as np
    import torch
    from paper_2511_10442_amd import binding as B
    from paper_2511_10442_amd import workloads as W

    dev = "cuda:0"
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
        ms = _timed(torch, lambda: B.fg_binned_select_knn(x, rs, k, 0, 0, ws, oi, od), args.reps)
        _, _, cand = B.fg_binned_select_knn_counted(x, rs, k, 0, 0, ws)
        torch.cuda.synchronize()
        cpq = float(cand.to(torch.float64).mean().item())
        nb, db = B.fg_auto_n_bins(n, 1, k, d, 1)
        brute = ""
        speed = ""
        if n <= 1_000_000:                                   # keep the brute-force leg bounded (about a second at 1M)
            ws1 = B.alloc_workspace(n, d, 1, k, 1, 2, dev)
            msb = _timed(torch, lambda: B.fg_binned_select_knn(x, rs, k, 1, 2, ws1, oi, od), 1 if n >= 1_000_000 else 2)
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
            f.write("Uniform random vectors, forward only, one MI355X; command: python bench.py --sweep uniform"
                    + (" --quick" if args.quick else "") + " --out " + args.out + "\n\n" + "\n".join(lines) + "\n")
    return 0


def run_profile_stage(args) -> int:
    import torch
    from paper_2511_10442_amd import binding as B
    from paper_2511_10442_amd import workloads as W

    dev = "cuda:0"
    if args.calib_mb > 0:
        a = torch.zeros(args.calib_mb * (1 << 20) // 4, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(args.reps):
            torch.add(a, 0.0, out=b)
        torch.cuda.synchronize()
    if args.profile_stage == "none":
        return 0
    if args.profile_stage == "oc":
        import numpy as np
        asso, uq, uqrs, rs_np, n_maxuq, n_maxrs = W.oc_association([100_000] * 10, 200, 0.1, seed=33)
        t = lambda arr: torch.from_numpy(np.ascontiguousarray(arr)).to(dev)
        A, U, R, S = t(asso), t(uq), t(uqrs), t(rs_np)
        M = torch.empty((n_maxuq, len(uq)), dtype=torch.int32, device=dev)
        Mn = torch.empty((n_maxrs, len(uq)), dtype=torch.int32, device=dev)
        wsp = torch.empty(B.fg_oc_helper_workspace_size(len(uq), n_maxrs), dtype=torch.uint8, device=dev)
        ms = _timed(torch, lambda: B.fg_oc_helper(A, U, R, S, n_maxuq, n_maxrs, True, 256, M, Mn, wsp), args.reps)
        out_bytes = (M.numel() + Mn.numel()) * 4
        print("fg_oc_helper: %.3f ms, n_unique=%d n_maxuq=%d n_maxrs=%d, %.0f MB written -> %.0f GB/s"
              % (ms, len(uq), n_maxuq, n_maxrs, out_bytes / 1e6, out_bytes / ms / 1e6))
        return 0
    w = W.CONFIGS[args.config]()
    wl = _Workload(torch, B, w, dev, args.n_bins, args.d_bin)
    k = w.k
    g = wl.g if wl.g is not None else torch.ones((w.n, k), device=dev)
    grad = wl.grad if wl.grad is not None else torch.empty((w.n, w.d), dtype=torch.float32, device=dev)
    if args.profile_stage == "query":
        bn = wl.bin()
        for _ in range(args.reps):
            B.fg_query_binned(bn, wl.rs, k, wl.out_idx, wl.out_d2)
    elif args.profile_stage == "forward":
        for _ in range(args.reps):
            B.fg_binned_select_knn(wl.x, wl.rs, k, args.n_bins, args.d_bin, wl.ws, wl.out_idx, wl.out_d2)
    elif args.profile_stage == "backward":
        B.fg_binned_select_knn(wl.x, wl.rs, k, args.n_bins, args.d_bin, wl.ws, wl.out_idx, wl.out_d2)
        for _ in range(args.reps):
            B.fg_knn_backward(g, wl.out_idx, wl.x, wl.rs, grad, wl.ws)
    else:                                                    # "step": what the default mode times
        for _ in range(args.reps):
            bn = wl.bin()
            B.fg_query_binned(bn, wl.rs, k, wl.out_idx, wl.out_d2)
            B.fg_knn_backward_binned(bn, g, wl.out_idx, wl.x, grad)
    torch.cuda.synchronize()
    print("profile stage done: config %d stage %s reps %d" % (args.config, args.profile_stage, args.reps))
    return 0


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
    ap.add_argument("--all-configs", action="store_true", help="add the stage table of all five configurations")
    ap.add_argument("--sweep", default="", choices=["", "uniform"])
    ap.add_argument("--quick", action="store_true", help="sweep: fewer and smaller points")
    ap.add_argument("--no-check", action="store_true", help="sweep: skip the oracle check of sampled rows")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--out", default="", help="sweep / --all-configs: also write the table to this file")
    ap.add_argument("--profile-stage", default="", choices=["", "query", "forward", "backward", "step", "oc", "none"])
    ap.add_argument("--calib-mb", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (segments are independent and would "
              "shard across GPUs with no exchange, but nothing here uses a second GPU); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if args.sweep:
        return run_sweep(args)
    if args.profile_stage:
        return run_profile_stage(args)
    return run_headline(args)


if __name__ == "__main__":
    sys.exit(main())
