"""Small driver for rocprofv3: runs one stage of the hot path a few times on a named workload.

    rocprofv3 --kernel-trace --stats -d <dir> -- python3 -m paper_2511_10442_amd.profile_run \
        --config 3 --stage query --reps 5

    --stage query     fg_bin_points once, then fg_query_binned `reps` times
    --stage forward   fg_binned_select_knn `reps` times
    --stage backward  forward once, then fg_knn_backward `reps` times
    --stage all       forward + backward `reps` times
    --stage oc        fg_oc_helper (Algorithm 3) `reps` times on 10 row splits of 100,000 vertices with 200
                      object candidates each; prints its mean time and output bandwidth
    --calib-mb M      additionally run one plain elementwise copy kernel (torch.add(a, 0, out=b))
                      over M MiB in and M MiB out, `reps` times: the known-size reference for
                      scaling memory counters
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--stage", default="query", choices=["query", "forward", "backward", "all", "oc", "none"])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--n-bins", type=int, default=0)
    ap.add_argument("--d-bin", type=int, default=0)
    ap.add_argument("--calib-mb", type=int, default=0)
    args = ap.parse_args()

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
    if args.stage == "none":
        return 0
    if args.stage == "oc":
        import numpy as np
        asso, uq, uqrs, rs_np, n_maxuq, n_maxrs = W.oc_association([100_000] * 10, 200, 0.1, seed=33)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        A, U, R, S = t(asso), t(uq), t(uqrs), t(rs_np)
        M = torch.empty((n_maxuq, len(uq)), dtype=torch.int32, device=dev)
        Mn = torch.empty((n_maxrs, len(uq)), dtype=torch.int32, device=dev)
        wsp = torch.empty(B.fg_oc_helper_workspace_size(len(uq), n_maxrs), dtype=torch.uint8, device=dev)
        B.fg_oc_helper(A, U, R, S, n_maxuq, n_maxrs, True, 256, M, Mn, wsp)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            B.fg_oc_helper(A, U, R, S, n_maxuq, n_maxrs, True, 256, M, Mn, wsp)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.reps
        out_bytes = (M.numel() + Mn.numel()) * 4
        print("fg_oc_helper: %.3f ms, n_unique=%d n_maxuq=%d n_maxrs=%d, %.0f MB written -> %.0f GB/s"
              % (ms, len(uq), n_maxuq, n_maxrs, out_bytes / 1e6, out_bytes / ms / 1e6))
        return 0
    w = W.CONFIGS[args.config]()
    x = torch.from_numpy(w.coords).to(dev)
    rs = torch.from_numpy(w.row_splits).to(dev)
    n, d, k, s = w.n, w.d, w.k, w.n_segments
    ws_bytes = max(B.fg_workspace_size(n, d, s, k, args.n_bins, args.d_bin), B.fg_workspace_size(n, d, s, k))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    out_idx = torch.empty((n, k), dtype=torch.int32, device=dev)
    out_d2 = torch.empty((n, k), dtype=torch.float32, device=dev)
    g = torch.from_numpy(w.grad_d2).to(dev) if w.grad_d2 is not None else torch.ones((n, k), device=dev)
    grad = torch.empty((n, d), dtype=torch.float32, device=dev)
    if args.stage == "query":
        bn = B.fg_bin_points(x, rs, k, args.n_bins, args.d_bin, ws)
        for _ in range(args.reps):
            B.fg_query_binned(bn, rs, k, out_idx, out_d2)
    elif args.stage == "forward":
        for _ in range(args.reps):
            B.fg_binned_select_knn(x, rs, k, args.n_bins, args.d_bin, ws, out_idx, out_d2)
    elif args.stage == "backward":
        B.fg_binned_select_knn(x, rs, k, args.n_bins, args.d_bin, ws, out_idx, out_d2)
        for _ in range(args.reps):
            B.fg_knn_backward(g, out_idx, x, rs, grad, ws)
    else:
        for _ in range(args.reps):
            B.fg_binned_select_knn(x, rs, k, args.n_bins, args.d_bin, ws, out_idx, out_d2)
            B.fg_knn_backward(g, out_idx, x, rs, grad, ws)
    torch.cuda.synchronize()
    print("profile_run done: config %d stage %s reps %d" % (args.config, args.stage, args.reps))
    return 0


if __name__ == "__main__":
    sys.exit(main())
