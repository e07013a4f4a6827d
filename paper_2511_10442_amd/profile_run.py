"""Small driver for rocprofv3: runs one stage of the hot path a few times on a named workload.

    rocprofv3 --kernel-trace --stats -d <dir> -- python3 -m paper_2511_10442_amd.profile_run \
        --config 3 --stage query --reps 5

    --stage query     fg_bin_points once, then fg_query_binned `reps` times
    --stage forward   fg_binned_select_knn `reps` times
    --stage backward  forward once, then fg_knn_backward `reps` times
    --stage all       forward + backward `reps` times
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
    ap.add_argument("--stage", default="query", choices=["query", "forward", "backward", "all", "none"])
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
