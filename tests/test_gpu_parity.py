"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs.  Indices and squared distances must be bit-exact; backward
gradients within 1e-5 relative (of the element's own scale, see `grad_close`)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_10442_amd import binding as B
from paper_2511_10442_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_knn(x, rs, k, n_bins=0, d_bin=0, counted=False):
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    rt = torch.from_numpy(np.ascontiguousarray(rs)).to(DEV)
    if counted:
        idx, d2, cand = B.fg_binned_select_knn_counted(xt, rt, k, n_bins, d_bin)
        torch.cuda.synchronize()
        return idx.cpu().numpy(), d2.cpu().numpy(), cand.cpu().numpy()
    idx, d2 = B.fg_binned_select_knn(xt, rt, k, n_bins, d_bin)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), d2.cpu().numpy()


def assert_exact(gi, gd, oi, od, what=""):
    bad_i = np.nonzero(gi != oi)
    assert bad_i[0].size == 0, "%s: %d index mismatches, first at row %d slot %d: got %d want %d" % (
        what, bad_i[0].size, bad_i[0][0], bad_i[1][0], gi[bad_i][0], oi[bad_i][0])
    bad_d = np.nonzero(gd.view(np.uint32) != od.view(np.uint32))
    assert bad_d[0].size == 0, "%s: %d distance mismatches, first at row %d slot %d: got %r want %r" % (
        what, bad_d[0].size, bad_d[0][0], bad_d[1][0], gd[bad_d][0], od[bad_d][0])


def check_against_oracle(x, rs, k, n_bins=0, d_bin=0, what=""):
    gi, gd = gpu_knn(x, rs, k, n_bins, d_bin)
    oi, od = oracle.knn(x, rs, k)
    assert_exact(gi, gd, oi, od, what)
    return gi, gd


def grad_close(g_gpu, g_ref, abs_sum, rtol=1e-5):
    """|G_gpu - G_ref| <= rtol * max(|G_ref|, A) per element, A = sum of |contributions| of that
    element (fp32 accumulation in any order cannot do better than a multiple of eps * A where
    terms cancel), and the max-norm error within rtol of the max-norm of the reference."""
    err = np.abs(g_gpu.astype(np.float64) - g_ref)
    scale = np.maximum(np.abs(g_ref), abs_sum)
    assert np.all(err <= rtol * scale + 1e-30), "max ratio %g" % np.max(err / (scale + 1e-30))
    assert err.max() <= rtol * max(np.abs(g_ref).max(), 1e-30)


# --------------------------------------------------------------------------- #
# small cases: several tiles of 64 queries + a ragged tail, every d, many k / n_bins / d_bin
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("d", list(range(2, 11)))
def test_uniform_every_dimension(d):
    sizes = [333, 0, 517, 64, 1, 150]
    x, rs = W.uniform(sum(sizes), d, seed=900 + d, sizes=sizes)
    for k, nb, db in [(8, 0, 0), (1, 0, 0), (17, 1, 2), (5, 7, min(d, 5)), (33, 3, 2), (64, 4, min(d, 3))]:
        check_against_oracle(x, rs, k, nb, db, "d=%d k=%d nb=%d db=%d" % (d, k, nb, db))


@pytest.mark.parametrize("k", [65, 66, 81, 97, 128])
def test_long_lists_two_passes(k):
    """More than 64 neighbours take two passes of the fast path (the second counts only keys above the
    first pass's last one): the boundary cases, heavy ties across the boundary, duplicates of the query,
    row splits shorter than K (padding in either pass), the candidate counts of both passes added up."""
    x, rs = W.quantised(2600, 3, 5, seed=1200 + k, sizes=[1500, 70, 0, 1000, 30])     # ~21 points per location
    check_against_oracle(x, rs, k, 0, 0, "quantised k=%d" % k)
    check_against_oracle(x, rs, k, 6, 3, "quantised k=%d nb=6" % k)
    x, rs = W.duplicates(1800, 2, 9, seed=1300 + k, sizes=[900, 900])                 # ~100 copies of each point
    check_against_oracle(x, rs, k, 0, 0, "duplicates k=%d" % k)
    x, rs = W.uniform(70_000, 3, seed=1400 + k, sizes=[40_000, 30_000])               # > 1024 tiles: ordered tiles
    gi, gd, cand = gpu_knn(x, rs, k, counted=True)
    rows = np.sort(np.random.Generator(np.random.PCG64(k)).choice(70_000, size=300, replace=False)).astype(np.int64)
    oi, od = oracle.knn_rows(x, rs, k, rows)
    assert_exact(gi[rows], gd[rows], oi, od, "uniform 70k k=%d" % k)
    assert cand.min() >= k - 1 and cand.max() < 70_000


@pytest.mark.parametrize("k", [2, 3, 16, 32, 40, 64, 100, 128])
def test_k_range(k):
    x, rs = W.uniform(1500, 3, seed=800 + k, sizes=[1000, 500])
    check_against_oracle(x, rs, k, 0, 0, "k=%d" % k)
    check_against_oracle(x, rs, k, 9, 3, "k=%d nb=9" % k)


@pytest.mark.parametrize("k", [16, 32, 48, 64])
def test_rows_written_from_registers_and_through_the_transposition(k):
    """Rows of exactly the list size leave the tile kernel as 16-byte stores when the output is
    16-byte aligned, through LDS otherwise: same result, nothing written outside the rows."""
    x, rs = W.uniform(2100, 3, seed=900 + k, sizes=[1500, 7, 593])          # a short split: padded rows
    n = x.shape[0]
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    oi, od = oracle.knn(x, rs, k)
    for shift in (0, 1):                                                     # shift 1: 4 bytes off alignment
        base_i = torch.full((n * k + 8,), -7, dtype=torch.int32, device=DEV)
        base_d = torch.full((n * k + 8,), -7.0, dtype=torch.float32, device=DEV)
        out_i = base_i[4 + shift:4 + shift + n * k].view(n, k)
        out_d = base_d[4 + shift:4 + shift + n * k].view(n, k)
        B.fg_binned_select_knn(xt, rt, k, 0, 0, None, out_i, out_d)
        torch.cuda.synchronize()
        assert_exact(out_i.cpu().numpy(), out_d.cpu().numpy(), oi, od, "k=%d shift=%d" % (k, shift))
        guard_i, guard_d = base_i.cpu().numpy(), base_d.cpu().numpy()
        assert np.all(guard_i[:4 + shift] == -7) and np.all(guard_i[4 + shift + n * k:] == -7)
        assert np.all(guard_d[:4 + shift] == -7.0) and np.all(guard_d[4 + shift + n * k:] == -7.0)


def test_n_bins_invariance():
    x, rs = W.uniform(3000, 3, seed=77, sizes=[1800, 1200])
    oi, od = oracle.knn(x, rs, 12)
    for nb, db in [(1, 2), (2, 3), (5, 3), (30, 3), (0, 0), (64, 3), (200, 2), (13, 2)]:
        gi, gd = gpu_knn(x, rs, 12, nb, db)
        assert_exact(gi, gd, oi, od, "nb=%d db=%d" % (nb, db))


def test_short_and_empty_segments_padding():
    sizes = [0, 3, 0, 0, 1, 9, 2, 0]
    x, rs = W.uniform(sum(sizes), 3, seed=5, sizes=sizes)
    gi, gd = check_against_oracle(x, rs, 6, 0, 0, "short segments")
    assert np.all(gi[0, 3:] == -1) and np.all(gd[0, 3:] == 0.0)
    check_against_oracle(x, rs, 6, 4, 2, "short segments nb=4")


def test_many_tiny_segments():
    sizes = W.ragged_sizes(400, 12, seed=9)
    x, rs = W.uniform(sum(sizes), 4, seed=10, sizes=sizes)
    check_against_oracle(x, rs, 5, 0, 0, "tiny segments")
    check_against_oracle(x, rs, 5, 3, 4, "tiny segments nb=3")


def test_duplicates_and_ties():
    x, rs = W.duplicates(2000, 3, n_distinct=37, seed=3, sizes=[1200, 800])
    check_against_oracle(x, rs, 20, 0, 0, "duplicates")
    check_against_oracle(x, rs, 20, 6, 3, "duplicates nb=6")
    x, rs = W.quantised(3000, 2, levels=9, seed=4, sizes=[3000])
    check_against_oracle(x, rs, 24, 0, 0, "quantised d=2")
    x, rs = W.quantised(3000, 5, levels=3, seed=6, sizes=[1000, 2000])
    check_against_oracle(x, rs, 24, 3, 5, "quantised d=5")


def test_all_identical_points():
    x = np.full((700, 3), -2.5, dtype=np.float32)
    rs = np.array([0, 300, 700], dtype=np.int32)
    check_against_oracle(x, rs, 9, 0, 0, "identical")
    check_against_oracle(x, rs, 9, 5, 3, "identical nb=5")


def test_lattice_and_collinear():
    x, rs = W.lattice(11, 3)
    check_against_oracle(x, rs, 27, 0, 0, "lattice 3d")
    check_against_oracle(x, rs, 27, 11, 3, "lattice 3d nb=11")
    x, rs = W.lattice(30, 2)
    check_against_oracle(x, rs, 13, 0, 0, "lattice 2d")
    x, rs = W.collinear(1000, 3)               # zero extent in two binning dimensions
    check_against_oracle(x, rs, 9, 0, 0, "collinear")
    check_against_oracle(x, rs, 9, 16, 3, "collinear nb=16")
    x, rs = W.collinear(1000, 4)
    x = np.ascontiguousarray(x[:, ::-1])       # the varying coordinate is the last (unbinned) one
    check_against_oracle(x, rs, 9, 8, 3, "collinear last dim")


def test_far_from_origin_and_tiny_scale():
    x, rs = W.uniform(2000, 3, seed=12, lo=1.0e6, hi=1.0e6 + 1.0)   # bin width below float spacing slack
    check_against_oracle(x, rs, 10, 0, 0, "offset 1e6")
    x, rs = W.uniform(2000, 3, seed=13, lo=-1e-18, hi=1e-18)        # squares around 1e-36..1e-37
    check_against_oracle(x, rs, 10, 0, 0, "scale 1e-18")
    x, rs = W.uniform(500, 2, seed=14, lo=0.0, hi=1e-20)            # denormal squared distances
    check_against_oracle(x, rs, 10, 0, 0, "scale 1e-20")
    x, rs = W.uniform(2000, 3, seed=15, lo=-1e15, hi=1e15)
    check_against_oracle(x, rs, 10, 0, 0, "scale 1e15")


def test_clustered_with_outliers():
    rng = np.random.Generator(np.random.PCG64(17))
    core = rng.standard_normal((3000, 3)) * 1e-3
    far = rng.random((40, 3)) * 100.0
    x = np.ascontiguousarray(np.concatenate([core, far]).astype(np.float32))
    rng.shuffle(x, axis=0)
    rs = np.array([0, x.shape[0]], dtype=np.int32)
    check_against_oracle(x, rs, 16, 0, 0, "cluster+outliers")
    check_against_oracle(x, rs, 16, 30, 3, "cluster+outliers nb=30")


def test_deterministic_across_runs():
    x, rs = W.uniform(5000, 3, seed=19)
    a = gpu_knn(x, rs, 16)
    b = gpu_knn(x, rs, 16)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_tile_and_list_kernels_both_run_and_agree_with_the_plain_walk():
    """Default path = tile kernel + list kernel for the queries it defers; algo = 1 sends
    every query through the one-lane-per-query walk.  Isolated points far from a dense core need
    many shells, so some queries must reach the list kernel."""
    rng = np.random.Generator(np.random.PCG64(29))
    core = rng.standard_normal((6000, 3)) * 0.05
    far = rng.random((600, 3)) * 20.0 - 10.0
    x = np.ascontiguousarray(np.concatenate([core, far]).astype(np.float32))
    rng.shuffle(x, axis=0)
    rs = np.array([0, 4000, x.shape[0]], dtype=np.int32)
    k = 12
    oi, od = oracle.knn(x, rs, k)
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    for nb in (0, 40):
        bn = B.fg_bin_points(xt, rt, k, nb, 3 if nb else 0)
        gi, gd = B.fg_query_binned(bn, rt, k)
        torch.cuda.synchronize()
        deferred = int(bn.work_count.item())
        assert_exact(gi.cpu().numpy(), gd.cpu().numpy(), oi, od, "tile+list nb=%d" % nb)
        assert 0 < deferred < x.shape[0]
        gi, gd = B.fg_query_binned(bn, rt, k, algo=1)
        torch.cuda.synchronize()
        assert_exact(gi.cpu().numpy(), gd.cpu().numpy(), oi, od, "plain walk nb=%d" % nb)


@pytest.mark.parametrize("d,k", [(2, 20), (3, 9), (3, 16), (3, 32), (3, 40), (3, 64), (4, 33), (5, 25), (6, 48), (8, 64), (10, 20),
                                 (3, 100), (3, 128)])
def test_flattened_scan_on_every_tile(d, k):
    """algo = 2: the tile kernel's flattened scan (the work of a chunk dealt out evenly over the lanes, kept
    candidates appended to their query's pending buffer from any lane) on every tile, for every list size and
    both passes of a long list.  Clustered points with duplicates, a short and an empty split, direction
    flags."""
    rng = np.random.Generator(np.random.PCG64(500 + 10 * d + k))
    sizes = [2300, 5, 0, 1700]
    n = sum(sizes)
    x, rs = W.uniform(n, d, seed=510 + d + k, sizes=sizes)
    x[100:400] = x[100]                                   # 300 copies of one point: ties on distance 0
    x[2400:3400] = x[2400] + 0.01 * (x[2400:3400] - 0.5)  # a dense cluster next to sparse points: uneven tiles
    x = np.ascontiguousarray(x)
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    oi, od = oracle.knn(x, rs, k)
    for nb in (0, 7):
        bn = B.fg_bin_points(xt, rt, k, nb, min(d, 3) if nb else 0)
        gi, gd = B.fg_query_binned(bn, rt, k, algo=2)
        torch.cuda.synchronize()
        assert_exact(gi.cpu().numpy(), gd.cpu().numpy(), oi, od, "flattened d=%d k=%d nb=%d" % (d, k, nb))
    direction = rng.integers(0, 4, size=n).astype(np.int32)
    oi, od = oracle.knn(x, rs, k, direction=direction)
    bn = B.fg_bin_points(xt, rt, k)
    dt = torch.from_numpy(direction).to(DEV)
    gi, gd = B.fg_query_binned(bn, rt, k, direction=dt, algo=2)
    torch.cuda.synchronize()
    assert_exact(gi.cpu().numpy(), gd.cpu().numpy(), oi, od, "flattened with flags d=%d k=%d" % (d, k))


def test_ordered_launch_takes_every_tile_once():
    """More than 1024 tiles: the ordering kernels rank the tiles by estimated work (heaviest first).  Every tile
    must still be taken exactly once: every row is compared with the plain walk, sampled rows with the oracle."""
    rng = np.random.Generator(np.random.PCG64(77))
    n, k = 90_000, 32
    centres = rng.random((40, 3)) * 10.0
    x = centres[rng.integers(0, 40, size=n)] + rng.standard_normal((n, 3)) * np.exp(rng.uniform(np.log(0.01), np.log(0.5), size=(n, 1)))
    x[:9000] = rng.random((9000, 3)) * 10.0
    x = np.ascontiguousarray(x.astype(np.float32))
    rs = np.array([0, 50_000, n], dtype=np.int32)
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    bn = B.fg_bin_points(xt, rt, k)
    gi, gd = B.fg_query_binned(bn, rt, k)
    torch.cuda.synchronize()
    assert (n + 63) // 64 > 1024
    rows = np.sort(rng.choice(n, size=3000, replace=False)).astype(np.int64)
    oi, od = oracle.knn_rows(x, rs, k, rows)
    gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
    assert np.array_equal(gi[rows], oi) and np.array_equal(gd[rows].view(np.uint32), od.view(np.uint32))
    gi1, gd1 = B.fg_query_binned(bn, rt, k, algo=1)                          # the plain walk agrees on every row
    torch.cuda.synchronize()
    assert np.array_equal(gi1.cpu().numpy(), gi) and np.array_equal(gd1.cpu().numpy().view(np.uint32), gd.view(np.uint32))


def gpu_knn_dir(x, rs, direction, k, n_bins=0, d_bin=0):
    idx, d2 = B.fg_binned_select_knn_dir(torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV),
                                         torch.from_numpy(direction).to(DEV), k, n_bins, d_bin)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), d2.cpu().numpy()


@pytest.mark.parametrize("d,k", [(2, 8), (3, 16), (3, 40), (5, 70), (4, 100)])
def test_direction_flags(d, k):
    """Algorithm 2's useDir / dir[]: 0 = neighbour only, 1 = query only, 2 = neither, else both."""
    sizes = [900, 0, 1500, 70, 3]
    n = sum(sizes)
    x, rs = W.uniform(n, d, seed=70 + d, sizes=sizes)
    rng = np.random.Generator(np.random.PCG64(71 + k))
    patterns = [rng.integers(0, 4, size=n), np.where(rng.random(n) < 0.9, 1, 0), np.ones(n), np.zeros(n),
                np.full(n, 2), np.full(n, 3), rng.integers(-3, 9, size=n)]
    for direction in patterns:
        direction = direction.astype(np.int32)
        oi, od = oracle.knn(x, rs, k, direction=direction)
        for nb, db in [(0, 0), (6, min(d, 3)), (1, 2)]:
            gi, gd = gpu_knn_dir(x, rs, direction, k, nb, db)
            assert_exact(gi, gd, oi, od, "dir d=%d k=%d nb=%d" % (d, k, nb))
    # plain walk kernel with flags
    direction = patterns[0].astype(np.int32)
    oi, od = oracle.knn(x, rs, k, direction=direction)
    xt, rt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    bn = B.fg_bin_points(xt, rt, k)
    dt = torch.from_numpy(direction).to(DEV)
    gi, gd = B.fg_query_binned(bn, rt, k, direction=dt, algo=1)
    torch.cuda.synchronize()
    assert_exact(gi.cpu().numpy(), gd.cpu().numpy(), oi, od, "dir plain walk")


def test_candidate_counts():
    """n_bins = 1: every query scans its whole row split minus itself (brute force through the
    same kernel); finer grids scan fewer candidates, never fewer than k-1."""
    sizes = [700, 300]
    x, rs = W.uniform(1000, 3, seed=23, sizes=sizes)
    gi, gd, cand = gpu_knn(x, rs, 8, 1, 2, counted=True)
    assert np.all(cand[:700] == 699) and np.all(cand[700:] == 299)
    gi2, gd2, cand2 = gpu_knn(x, rs, 8, 6, 3, counted=True)
    assert_exact(gi2, gd2, gi, gd)
    assert np.all(cand2 >= 7) and cand2.sum() < cand.sum()


# --------------------------------------------------------------------------- #
# binning stage invariants
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("d,nb,db", [(3, 0, 0), (3, 7, 3), (2, 30, 2), (6, 4, 5), (4, 1, 2)])
def test_binning_invariants(d, nb, db):
    sizes = [2000, 0, 1234, 1]
    n = sum(sizes)
    x, rs = W.uniform(n, d, seed=31 + d, sizes=sizes)
    xt = torch.from_numpy(x).to(DEV)
    rt = torch.from_numpy(rs).to(DEV)
    bn = B.fg_bin_points(xt, rt, 8, nb, db)
    torch.cuda.synchronize()
    perm = bn.perm.cpu().numpy()
    bounds = bn.bin_bounds.cpu().numpy()
    bin_idx = bn.bin_idx.cpu().numpy()
    rec = bn.sorted_records.cpu().numpy()
    geom = bn.seg_geom.cpu().numpy()
    T = bn.cells_per_segment
    assert sorted(perm.tolist()) == list(range(n))                       # a permutation
    assert bounds[0] == 0 and bounds[-1] == n and np.all(np.diff(bounds) >= 0)
    for s in range(len(sizes)):                                          # segment s owns bins [sT, (s+1)T)
        assert bounds[s * T] == rs[s] and bounds[(s + 1) * T] == rs[s + 1]
    sorted_bins = bin_idx[perm]
    assert np.all(np.diff(sorted_bins) >= 0)                             # sorted by bin
    assert np.array_equal(np.bincount(bin_idx, minlength=len(bounds) - 1), np.diff(bounds))
    assert np.array_equal(rec[:, :d], x[perm])                           # coordinates moved with their points
    assert rec.shape[1] == (d + 1 + 3) // 4 * 4 and np.all(rec[:, d + 1:] == 0.0)
    # the box is the row split's true bounding box; every point's bin is inside its own segment's range
    seg = np.searchsorted(rs[1:], np.arange(n), side="right")
    assert np.all(bin_idx // T == seg)
    for s, size in enumerate(sizes):
        if size > 1:
            assert np.array_equal(geom[s, :, 0], x[rs[s]:rs[s + 1], :bn.d_bin].min(axis=0))
    # bins are monotone in every binned coordinate (what the search's lower bounds rely on)
    local = bin_idx - seg * T
    assert T == bn.n_bins ** bn.d_bin * bn.sub_bins and bn.sub_bins in (1, 2, 4)
    last = bn.n_bins * bn.sub_bins                                        # cells along the last binning dimension
    for c in range(bn.d_bin):
        cell_c = local % last if c == bn.d_bin - 1 else (local // (last * bn.n_bins ** (bn.d_bin - 2 - c))) % bn.n_bins
        for s, size in enumerate(sizes):
            if size > 1:
                sl = slice(rs[s], rs[s + 1])
                order = np.argsort(x[sl, c], kind="stable")
                assert np.all(np.diff(cell_c[sl][order]) >= 0)


# --------------------------------------------------------------------------- #
# backward
# --------------------------------------------------------------------------- #
def gpu_backward(g, idx, x, rs=None):
    """rs given: bin-ordered kernel that combines contributions in LDS; None: plain atomic scatter."""
    out = B.fg_knn_backward(torch.from_numpy(g).to(DEV), torch.from_numpy(idx).to(DEV),
                            torch.from_numpy(x).to(DEV),
                            None if rs is None else torch.from_numpy(rs).to(DEV))
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("d,k", [(2, 16), (3, 5), (4, 40), (7, 33), (10, 128)])
def test_backward_small(d, k):
    sizes = [700, 3, 0, 500]
    n = sum(sizes)
    x, rs = W.uniform(n, d, seed=41 + d, sizes=sizes)
    idx, _ = oracle.knn(x, rs, k)                 # includes -1 padding in the 3-point split
    g = W.upstream_grad(n, k, seed=43)
    ref, asum = oracle.knn_backward(g, idx, x)
    grad_close(gpu_backward(g, idx, x), ref, asum)
    grad_close(gpu_backward(g, idx, x, rs), ref, asum)


@pytest.mark.parametrize("d,k", [(2, 16), (3, 32), (5, 40), (8, 7)])
def test_backward_on_the_forward_binning(d, k):
    """Bin once, query, backward in the same bin order: the gradient of the graph just built."""
    sizes = [900, 2, 1300]
    n = sum(sizes)
    x, rs = W.uniform(n, d, seed=71 + d, sizes=sizes)
    xt, rst = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV)
    ws = B.alloc_workspace(n, d, len(sizes), k, 0, 0, DEV)
    binning = B.fg_bin_points(xt, rst, k, 0, 0, ws)
    gi, gd = B.fg_query_binned(binning, rst, k)
    g = W.upstream_grad(n, k, seed=73)
    out = B.fg_knn_backward_binned(binning, torch.from_numpy(g).to(DEV), gi, xt)
    torch.cuda.synchronize()
    oi, _ = oracle.knn(x, rs, k)
    assert np.array_equal(gi.cpu().numpy(), oi)
    ref, asum = oracle.knn_backward(g, oi, x)
    grad_close(out.cpu().numpy(), ref, asum)


def test_backward_hash_table_overflow_and_hot_destination():
    """More distinct destinations per block than the LDS table holds (random far neighbours), and one
    destination shared by every row: both must still add up."""
    n, k, d = 6000, 64, 3
    x, rs = W.uniform(n, d, seed=61)
    rng = np.random.Generator(np.random.PCG64(62))
    idx = rng.integers(0, n, size=(n, k)).astype(np.int32)
    idx[:, 5] = 17
    idx[rng.random((n, k)) < 0.05] = -1
    g = W.upstream_grad(n, k, seed=63)
    ref, asum = oracle.knn_backward(g, idx, x)
    grad_close(gpu_backward(g, idx, x, rs), ref, asum)
    grad_close(gpu_backward(g, idx, x), ref, asum)


def test_backward_overwrites_and_ignores_padding():
    x, rs = W.uniform(100, 3, seed=51)
    idx = np.full((100, 4), -1, dtype=np.int32)
    g = W.upstream_grad(100, 4, seed=52)
    out = B.fg_knn_backward(torch.from_numpy(g).to(DEV), torch.from_numpy(idx).to(DEV),
                            torch.from_numpy(x).to(DEV), None,
                            torch.full((100, 3), 7.0, dtype=torch.float32, device=DEV))
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 0.0)
    out = B.fg_knn_backward(torch.from_numpy(g).to(DEV), torch.from_numpy(idx).to(DEV),
                            torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV),
                            torch.full((100, 3), 7.0, dtype=torch.float32, device=DEV))
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 0.0)


def test_forward_and_backward_replay_in_a_hip_graph():
    """The library enqueues only kernels (counters are cleared by fill kernels, not memset nodes) and never
    synchronises or allocates, so a whole step can be captured once and replayed.  Every replay is checked
    against the oracle, with eager work and synchronisations in between."""
    x, rs = W.uniform(20000, 3, seed=91, sizes=[12000, 8000])
    k = 16
    g = W.upstream_grad(20000, k, seed=92)
    oi, od = oracle.knn(x, rs, k)
    ref, asum = oracle.knn_backward(g, oi, x)
    xt, rt, gt = torch.from_numpy(x).to(DEV), torch.from_numpy(rs).to(DEV), torch.from_numpy(g).to(DEV)
    ws = B.alloc_workspace(20000, 3, 2, k, 0, 0, DEV)
    out_i = torch.empty((20000, k), dtype=torch.int32, device=DEV)
    out_d = torch.empty((20000, k), dtype=torch.float32, device=DEV)
    grad = torch.empty((20000, 3), dtype=torch.float32, device=DEV)

    def step():
        B.fg_binned_select_knn(xt, rt, k, 0, 0, ws, out_i, out_d)
        B.fg_knn_backward(gt, out_i, xt, rt, grad, ws)

    step()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        out_i.fill_(-7)
        out_d.fill_(-1.0)
        grad.fill_(5.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_exact(out_i.cpu().numpy(), out_d.cpu().numpy(), oi, od, "graph replay %d" % rep)
        grad_close(grad.cpu().numpy(), ref, asum)
        junk = (xt * 2.0).sum().item()       # eager work between the replays
        assert junk == junk
