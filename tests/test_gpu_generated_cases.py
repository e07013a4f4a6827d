"""GPU parity on generated cases: hypothesis draws the shape of the problem (dimension, K, ragged row splits
with empty ones, the value distribution, the grid), the points themselves come from the seeded generators, and
the HIP path must match the oracle bit for bit, forward, and within the gradient tolerance, backward.
The examples are derandomised: every run sees the same cases."""
import numpy as np
import pytest
import torch
from hypothesis import given, settings, HealthCheck, strategies as st

import oracle
from paper_2511_10442_amd import binding as B
from paper_2511_10442_amd import workloads as W
from test_gpu_parity import assert_exact, grad_close, gpu_knn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

sizes_st = st.lists(st.one_of(st.just(0), st.integers(1, 3), st.integers(4, 400), st.integers(400, 2500)),
                    min_size=1, max_size=6).filter(lambda s: 0 < sum(s) <= 6000)


def points(kind, n, d, seed, sizes):
    if kind == "uniform":
        return W.uniform(n, d, seed=seed, sizes=sizes)
    if kind == "shifted":                                   # far from the origin: coarse float grid, many ties
        x, rs = W.uniform(n, d, seed=seed, lo=4096.0, hi=4097.0, sizes=sizes)
        return x, rs
    if kind == "quantised":
        return W.quantised(n, d, 4, seed=seed, sizes=sizes)
    if kind == "duplicates":
        return W.duplicates(n, d, max(1, n // 40), seed=seed, sizes=sizes)
    x, rs = W.uniform(n, d, seed=seed, sizes=sizes)         # "flat": no extent in the last binning dimensions
    x[:, 1:] = 0.25
    return x, rs


@settings(max_examples=800, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
@given(d=st.integers(2, 10), k=st.one_of(st.integers(1, 70), st.sampled_from([16, 32, 48, 64, 65, 128])),
       sizes=sizes_st, kind=st.sampled_from(["uniform", "shifted", "quantised", "duplicates", "flat"]),
       grid=st.sampled_from([(0, 0), (0, 2), (1, 2), (3, 2), (5, 3), (9, 4), (12, 5), (40, 2)]),
       seed=st.integers(0, 2 ** 16))
def test_forward_generated(d, k, sizes, kind, grid, seed):
    n = sum(sizes)
    x, rs = points(kind, n, d, seed, sizes)
    nb, db = grid
    db = min(db, d, 5) if db else 0
    gi, gd = gpu_knn(x, rs, k, nb, db)
    oi, od = oracle.knn(x, rs, k)
    assert_exact(gi, gd, oi, od, "d=%d k=%d sizes=%s %s grid=%s seed=%d" % (d, k, sizes, kind, grid, seed))


@settings(max_examples=80, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
@given(d=st.integers(2, 10), k=st.integers(1, 70), sizes=sizes_st,
       kind=st.sampled_from(["uniform", "quantised", "duplicates"]), binned=st.booleans(), seed=st.integers(0, 2 ** 16))
def test_backward_generated(d, k, sizes, kind, binned, seed):
    n = sum(sizes)
    x, rs = points(kind, n, d, seed, sizes)
    idx, _ = oracle.knn(x, rs, k)
    g = W.upstream_grad(n, k, seed=seed + 1)
    ref, abs_sum = oracle.knn_backward(g, idx, x)
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    gt, it = torch.from_numpy(g).to(DEV), torch.from_numpy(idx).to(DEV)
    if binned:
        bn = B.fg_bin_points(xt, rt, k)
        out = B.fg_knn_backward_binned(bn, gt, it, xt)
    else:
        out = B.fg_knn_backward(gt, it, xt, rt)
    torch.cuda.synchronize()
    grad_close(out.cpu().numpy(), ref, abs_sum)
