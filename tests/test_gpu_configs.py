"""GPU parity at the five full-size configurations, in the launch configuration bench.py times
(automatic bins).  Small configurations are compared with the full oracle result; the large
ones on (i) sampled rows the oracle computes one by one, (ii) per-block digests of the full
oracle result where a digest file was precomputed on the CPU (tests/golden/), and (iii)
properties that hold at any size.  Backward is compared with the double-precision oracle."""
import hashlib
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2511_10442_amd import binding as B
from paper_2511_10442_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
BLOCK = 4096
_cache = {}


def workload(cfg):
    if cfg not in _cache:
        _cache.clear()                      # keep at most one large workload alive
        _cache[cfg] = W.CONFIGS[cfg]()
    return _cache[cfg]


def forward(w, n_bins=0, d_bin=0):
    x = torch.from_numpy(w.coords).to(DEV)
    rs = torch.from_numpy(w.row_splits).to(DEV)
    idx, d2 = B.fg_binned_select_knn(x, rs, w.k, n_bins, d_bin)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), d2.cpu().numpy()


def assert_rows_exact(gi, gd, oi, od, rows, what):
    bad = np.nonzero(np.any(gi[rows] != oi, axis=1) | np.any(gd[rows].view(np.uint32) != od.view(np.uint32), axis=1))[0]
    assert bad.size == 0, "%s: %d of %d sampled rows differ, first row %d: got %s / %s want %s / %s" % (
        what, bad.size, len(rows), rows[bad[0]], gi[rows[bad[0]]], gd[rows[bad[0]]], oi[bad[0]], od[bad[0]])


def check_properties(w, gi, gd):
    """Properties of the exact graph that hold at any size (Algorithm 2: slot 0 is the query at
    distance 0, the query is not its own candidate, searches stay inside the row split) plus
    ordering, and bit-exact recomputation of every returned distance from its index."""
    n, k = gi.shape
    assert np.array_equal(gi[:, 0], np.arange(n, dtype=np.int32)) and np.all(gd[:, 0] == 0.0)
    seg = np.searchsorted(w.row_splits[1:], np.arange(n), side="right")
    valid = gi >= 0
    sizes = np.diff(w.row_splits)[seg]
    assert np.array_equal(valid.sum(axis=1), np.minimum(sizes, k))          # padded only when the split is short
    nb_seg = np.searchsorted(w.row_splits[1:], np.where(valid, gi, 0), side="right")
    assert np.all((nb_seg == seg[:, None]) | ~valid)
    assert np.all((gi[:, 1:] != gi[:, :1]) | ~valid[:, 1:])                 # self only at slot 0
    a_d, b_d, a_i, b_i = gd[:, 1:-1], gd[:, 2:], gi[:, 1:-1], gi[:, 2:]
    ok = (a_d < b_d) | ((a_d == b_d) & (a_i < b_i)) | (b_i < 0)
    assert np.all(ok)                                                       # strictly ascending (d2, index)
    # distances recomputed in float32, one rounded operation at a time, left to right
    x = w.coords
    for j in range(1, k):
        u = np.where(valid[:, j], gi[:, j], np.arange(n))
        acc = None
        for c in range(x.shape[1]):
            delta = x[:, c] - x[u, c]
            sq = delta * delta
            acc = sq if acc is None else acc + sq
        acc = np.where(valid[:, j], acc, np.float32(0.0)).astype(np.float32)
        assert np.array_equal(acc.view(np.uint32), gd[:, j].view(np.uint32)), "slot %d" % j


def check_digests(cfg, gi, gd, seg=None):
    """Every row of the run against the oracle's complete result, through per-block digests written on the CPU by
    tests/golden/make_config_digests.py.  The digest file must exist."""
    name = "config%d_digests.txt" % cfg if seg is None else "config%d_seg%d_digests.txt" % (cfg, seg)
    path = os.path.join(GOLDEN, name)
    assert os.path.exists(path), "missing oracle digests %s" % name
    want = [l.strip() for l in open(path) if l.strip() and not l.startswith("#")]
    w = workload(cfg)
    b0, e0 = (0, w.n) if seg is None else (int(w.row_splits[seg]), int(w.row_splits[seg + 1]))
    got = []
    for b in range(b0, e0, BLOCK):
        h = hashlib.blake2b(digest_size=8)
        h.update(np.ascontiguousarray(gi[b:min(b + BLOCK, e0)]).tobytes())
        h.update(np.ascontiguousarray(gd[b:min(b + BLOCK, e0)]).tobytes())
        got.append(h.hexdigest())
    bad = [i for i, (g, o) in enumerate(zip(got, want)) if g != o]
    assert len(got) == len(want) and not bad, "config %d: %d of %d blocks differ from the oracle digests, first block %d" % (
        cfg, len(bad), len(want), bad[0] if bad else -1)


def sample_rows(n, count, seed):
    rows = np.random.Generator(np.random.PCG64(seed)).choice(n, size=min(count, n), replace=False)
    return np.sort(rows).astype(np.int64)


def grad_close(g_gpu, g_ref, abs_sum, rtol=1e-5):
    err = np.abs(g_gpu.astype(np.float64) - g_ref)
    scale = np.maximum(np.abs(g_ref), abs_sum)
    assert np.all(err <= rtol * scale + 1e-30), "max ratio %g" % np.max(err / (scale + 1e-30))
    assert err.max() <= rtol * max(np.abs(g_ref).max(), 1e-30)


def backward_gpu(g, idx, x, rs):
    out = B.fg_knn_backward(torch.from_numpy(g).to(DEV), torch.from_numpy(np.ascontiguousarray(idx)).to(DEV),
                            torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def backward_binned_gpu(g, idx, x, rs, k):
    """The bench's launch configuration: backward in the bin order of the forward's binning."""
    xt, rst = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    ws = B.alloc_workspace(x.shape[0], x.shape[1], len(rs) - 1, k, 0, 0, DEV)
    binning = B.fg_bin_points(xt, rst, k, 0, 0, ws)
    out = B.fg_knn_backward_binned(binning, torch.from_numpy(g).to(DEV),
                                   torch.from_numpy(np.ascontiguousarray(idx)).to(DEV), xt)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def sampled_graph(w, rows):
    """[n,k] index matrix whose sampled rows are the oracle's neighbours and every other row is padding."""
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    idx = np.full((w.n, w.k), -1, dtype=np.int32)
    idx[rows] = oi
    return idx, oi, od


def random_in_segment_graph(w, seed):
    """Dense synthetic index matrix: every entry a random point of the row's own split (some -1)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    seg = np.searchsorted(w.row_splits[1:], np.arange(w.n), side="right")
    lo = w.row_splits[:-1][seg].astype(np.int64)
    size = np.diff(w.row_splits)[seg].astype(np.int64)
    idx = (lo[:, None] + (rng.random((w.n, w.k)) * size[:, None]).astype(np.int64)).astype(np.int32)
    idx[rng.random((w.n, w.k)) < 0.02] = -1
    return idx


# --------------------------------------------------------------------------- #
def test_config1_full():
    w = workload(1)
    gi, gd = forward(w)
    oi, od = oracle.knn(w.coords, w.row_splits, w.k)
    assert np.array_equal(gi, oi) and np.array_equal(gd.view(np.uint32), od.view(np.uint32))
    check_properties(w, gi, gd)
    nb, db = B.fg_auto_n_bins(w.n, 1, w.k, 3, mode=0)           # the paper's own bin count
    gi2, gd2 = forward(w, nb, db)
    assert np.array_equal(gi2, oi) and np.array_equal(gd2.view(np.uint32), od.view(np.uint32))


def test_config2_full_forward_and_backward():
    w = workload(2)
    gi, gd = forward(w)
    oi, od = oracle.knn(w.coords, w.row_splits, w.k)
    assert np.array_equal(gi, oi) and np.array_equal(gd.view(np.uint32), od.view(np.uint32))
    check_properties(w, gi, gd)
    ref, asum = oracle.knn_backward(w.grad_d2, oi, w.coords)
    grad_close(backward_gpu(w.grad_d2, oi, w.coords, w.row_splits), ref, asum)
    grad_close(backward_binned_gpu(w.grad_d2, oi, w.coords, w.row_splits, w.k), ref, asum)
    nb, db = B.fg_auto_n_bins(w.n, w.n_segments, w.k, w.d, mode=0)   # paper: 14 bins over 4 dims
    gi2, gd2 = forward(w, nb, db)
    assert np.array_equal(gi2, oi) and np.array_equal(gd2.view(np.uint32), od.view(np.uint32))


def test_config3_forward():
    w = workload(3)
    gi, gd = forward(w)
    check_properties(w, gi, gd)
    rows = sample_rows(w.n, 6000, seed=303)
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "config 3")
    check_digests(3, gi, gd)
    gi2, gd2 = forward(w, 30, 3)                                 # the paper's clamped bin count
    assert np.array_equal(gi2, gi) and np.array_equal(gd2.view(np.uint32), gd.view(np.uint32))
    # the two calls bench.py times (bin, then query on that binning)
    xt, rst = torch.from_numpy(w.coords).to(DEV), torch.from_numpy(w.row_splits).to(DEV)
    ws = B.alloc_workspace(w.n, w.d, w.n_segments, w.k, 0, 0, DEV)
    gi3, gd3 = B.fg_query_binned(B.fg_bin_points(xt, rst, w.k, 0, 0, ws), rst, w.k)
    torch.cuda.synchronize()
    assert np.array_equal(gi3.cpu().numpy(), gi) and np.array_equal(gd3.cpu().numpy().view(np.uint32), gd.view(np.uint32))


def real_graph_backward(cfg):
    """The flow bench.py times, at full size: forward on the GPU (the index matrix is checked against the oracle's
    digests first, so it IS the oracle's graph), then both backward entry points on that graph against the
    double-precision oracle backward of the same matrix."""
    w = workload(cfg)
    gi, gd = forward(w)
    if cfg == 5:
        for seg in range(w.n_segments):
            check_digests(5, gi, gd, seg=seg)
    else:
        check_digests(cfg, gi, gd)
    ref, asum = oracle.knn_backward(w.grad_d2, gi, w.coords)
    assert np.abs(ref).max() > 0
    grad_close(backward_binned_gpu(w.grad_d2, gi, w.coords, w.row_splits, w.k), ref, asum)
    grad_close(backward_gpu(w.grad_d2, gi, w.coords, w.row_splits), ref, asum)


def test_config3_backward_on_the_real_graph():
    real_graph_backward(3)


def test_config3_backward():
    w = workload(3)
    rows = sample_rows(w.n, 20000, seed=313)
    idx, _, _ = sampled_graph(w, rows)
    ref, asum = oracle.knn_backward(w.grad_d2, idx, w.coords)
    grad_close(backward_gpu(w.grad_d2, idx, w.coords, w.row_splits), ref, asum)
    grad_close(backward_binned_gpu(w.grad_d2, idx, w.coords, w.row_splits, w.k), ref, asum)
    idx = random_in_segment_graph(w, seed=323)
    ref, asum = oracle.knn_backward(w.grad_d2, idx, w.coords)
    grad_close(backward_gpu(w.grad_d2, idx, w.coords, w.row_splits), ref, asum)
    grad_close(backward_binned_gpu(w.grad_d2, idx, w.coords, w.row_splits, w.k), ref, asum)


def test_config4_forward():
    w = workload(4)
    gi, gd = forward(w)
    check_properties(w, gi, gd)
    rows = sample_rows(w.n, 1500, seed=404)
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "config 4")
    check_digests(4, gi, gd)


def test_config4_paper_bins():
    w = workload(4)
    nb, db = B.fg_auto_n_bins(w.n, 1, w.k, w.d, mode=0)          # paper: 12 bins over the first 5 dims
    assert (nb, db) == (12, 5)
    gi, gd = forward(w, nb, db)
    rows = sample_rows(w.n, 1500, seed=414)
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "config 4, 12 bins x 5 dims")


def test_config5_forward():
    w = workload(5)
    gi, gd = forward(w)
    check_properties(w, gi, gd)
    rows = sample_rows(w.n, 3000, seed=505)
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "config 5")
    for seg in range(w.n_segments):
        check_digests(5, gi, gd, seg=seg)
    # the densest spot: points closest to the origin of the first split
    r2 = np.sum(w.coords[: w.row_splits[1]].astype(np.float64) ** 2, axis=1)
    rows = np.sort(np.argsort(r2)[:300]).astype(np.int64)
    oi, od = oracle.knn_rows(w.coords, w.row_splits, w.k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "config 5 centre")


def test_config5_backward_on_the_real_graph():
    real_graph_backward(5)


def test_config5_backward():
    w = workload(5)
    rows = sample_rows(w.n, 8000, seed=515)
    idx, _, _ = sampled_graph(w, rows)
    ref, asum = oracle.knn_backward(w.grad_d2, idx, w.coords)
    grad_close(backward_gpu(w.grad_d2, idx, w.coords, w.row_splits), ref, asum)
    idx = random_in_segment_graph(w, seed=525)
    ref, asum = oracle.knn_backward(w.grad_d2, idx, w.coords)
    grad_close(backward_gpu(w.grad_d2, idx, w.coords, w.row_splits), ref, asum)
    _cache.clear()


@pytest.mark.parametrize("d", [2, 5, 8])
def test_uniform_sweep_points_at_one_million(d):
    """Three points of the uniform sweep (the paper's own benchmark shape, Section 4: 1M uniform random vectors,
    K = 40) at full size in the launch configuration bench.py --sweep uniform times: sampled rows against the
    oracle, every row against the size-independent properties."""
    _cache.clear()
    x, rs = W.uniform(1_000_000, d, seed=4000 + d)
    k = 40
    idx, d2 = B.fg_binned_select_knn(torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV), k)
    torch.cuda.synchronize()
    gi, gd = idx.cpu().numpy(), d2.cpu().numpy()
    rows = sample_rows(x.shape[0], 400, seed=600 + d)
    oi, od = oracle.knn_rows(x, rs, k, rows)
    assert_rows_exact(gi, gd, oi, od, rows, "uniform 1M d=%d" % d)

    class _W:
        coords, row_splits = x, rs
    check_properties(_W, gi, gd)


def test_output_larger_than_two_to_the_31_elements():
    """The maximum-size case the interface allows in this memory: n * K beyond 2^31 output elements (row offsets must
    be 64-bit everywhere) with a two-pass list (K - 1 > 64) over two row splits; forward rows sampled across the
    whole range against the oracle, backward checked for the rows whose gradient the sample determines."""
    n, d, k = 20_000_000, 3, 108
    assert n * k > 2 ** 31
    rng = np.random.Generator(np.random.PCG64(77))
    x = rng.random((n, d), dtype=np.float32)
    rs = np.array([0, n // 3, n], dtype=np.int32)
    xt = torch.from_numpy(x).to(DEV)
    rt = torch.from_numpy(rs).to(DEV)
    idx, d2 = B.fg_binned_select_knn(xt, rt, k)
    torch.cuda.synchronize()
    rows = np.sort(np.concatenate([rng.choice(n, size=60, replace=False), [0, n // 3 - 1, n // 3, n - 1]])).astype(np.int64)
    oi, od = oracle.knn_rows(x, rs, k, rows)
    sel = torch.from_numpy(rows).to(DEV)
    gi, gd = idx[sel].cpu().numpy(), d2[sel].cpu().numpy()
    assert np.array_equal(gi, oi)
    assert np.array_equal(gd.view(np.uint32), od.view(np.uint32))
    # backward: a gradient only on the sampled rows' entries touches the sampled rows and their neighbours
    g = torch.zeros((n, k), dtype=torch.float32, device=DEV)
    g_rows = torch.from_numpy(rng.standard_normal((len(rows), k)).astype(np.float32)).to(DEV)
    g[sel] = g_rows
    grad = B.fg_knn_backward(g, idx, xt, rt)
    torch.cuda.synchronize()
    ref = {}
    gr = g_rows.cpu().numpy().astype(np.float64)
    for i, v in enumerate(rows):
        for j in range(k):
            u = int(oi[i, j])
            if u < 0 or u == v:
                continue
            t = 2.0 * gr[i, j] * (x[v].astype(np.float64) - x[u].astype(np.float64))
            ref[int(v)] = ref.get(int(v), 0.0) + t
            ref[u] = ref.get(u, 0.0) - t
    touched = np.array(sorted(ref.keys()), dtype=np.int64)
    got = grad[torch.from_numpy(touched).to(DEV)].cpu().numpy().astype(np.float64)
    want = np.stack([ref[int(t)] for t in touched])
    scale = np.abs(want).max()
    assert np.abs(got - want).max() <= 1e-5 * scale
    assert float(grad.abs().sum().item()) > 0.0
    total = float(grad.double().abs().sum().item())
    assert abs(total - np.abs(got).sum()) <= 1e-6 * total       # nothing outside the touched rows
