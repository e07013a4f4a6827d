"""Seeded synthetic inputs for the binned exact kNN path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no distances, no binning, no selection).  Both the CPU
oracle and the HIP path are fed the arrays produced here, so it imports neither.

All generators use ``numpy.random.Generator(PCG64(seed))``, do their math in
float64 and cast once to float32.  The five configurations are the workloads the
build is measured and parity-checked on; the paper itself benchmarks on uniformly
distributed random vectors of 1e3..5e6 points (Section 4, first paragraph), and
motivates the method with clustered low-dimensional detector-hit clouds
(Abstract; Section 5), which configurations 2, 3 and 5 stand in for.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class Workload:
    name: str
    coords: np.ndarray          # [N, d] float32, C-contiguous
    row_splits: np.ndarray      # [S+1] int32, row_splits[0]=0, row_splits[S]=N
    k: int
    n_bins: int = 0             # <=0: let the library choose
    d_bin: int = 0              # <=0: let the library choose
    backward: bool = False
    grad_d2: Optional[np.ndarray] = None   # [N, k] float32 upstream gradient
    note: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.coords.shape[0])

    @property
    def d(self) -> int:
        return int(self.coords.shape[1])

    @property
    def n_segments(self) -> int:
        return int(self.row_splits.shape[0] - 1)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.astype(np.float32))


def _splits(sizes) -> np.ndarray:
    rs = np.zeros(len(sizes) + 1, dtype=np.int64)
    rs[1:] = np.cumsum(np.asarray(sizes, dtype=np.int64))
    assert rs[-1] < 2**31
    return rs.astype(np.int32)


def upstream_grad(n: int, k: int, seed: int) -> np.ndarray:
    """Upstream gradient on the squared distances, i.i.d. N(0,1), float32 [n,k]."""
    return _f32(_rng(seed).standard_normal((n, k)))


# --------------------------------------------------------------------------- #
# the five configurations
# --------------------------------------------------------------------------- #

def config1(n: int = 4096, k: int = 16, seed: int = 1001) -> Workload:
    """Single segment, d=3, i.i.d. uniform [0,1); forward only."""
    x = _rng(seed).random((n, 3))
    return Workload("C1_uniform_d3", _f32(x), _splits([n]), k,
                    note="N=%d d=3 U[0,1) k=%d single segment" % (n, k))


def config2(n_per_segment: int = 50_000, n_segments: int = 2, k: int = 40,
            seed: int = 1002, grad_seed: int = 2002) -> Workload:
    """d=4 mixture of 50 isotropic Gaussians (sigma 0.3, means U[0,10]^4, shared by
    the segments) + 10 % uniform background; forward + backward."""
    rng = _rng(seed)
    means = rng.random((50, 4)) * 10.0
    n_bg = n_per_segment // 10
    n_cl = n_per_segment - n_bg
    parts = []
    for _ in range(n_segments):
        which = rng.integers(0, 50, size=n_cl)
        cl = means[which] + 0.3 * rng.standard_normal((n_cl, 4))
        bg = rng.random((n_bg, 4)) * 10.0
        seg = np.concatenate([cl, bg], axis=0)
        rng.shuffle(seg, axis=0)
        parts.append(seg)
    x = _f32(np.concatenate(parts, axis=0))
    n = x.shape[0]
    return Workload("C2_gauss_mix_d4", x, _splits([n_per_segment] * n_segments), k,
                    backward=True, grad_d2=upstream_grad(n, k, grad_seed),
                    note="N=%d d=4 50 Gaussians sigma=0.3 + 10%% uniform, %d segments, k=%d"
                         % (n, n_segments, k))


def _shower_segment(rng: np.random.Generator, n_points: int, n_showers: int,
                    mean_size: float) -> np.ndarray:
    chunks = []
    for _ in range(n_showers):
        centre = rng.random(3) * 10.0
        sig = np.exp(rng.uniform(np.log(0.01), np.log(0.5), size=3))
        q, r = np.linalg.qr(rng.standard_normal((3, 3)))
        q = q * np.sign(np.diag(r))          # sign-fixed rotation/reflection basis
        m = int(rng.poisson(mean_size))
        pts = (rng.standard_normal((m, 3)) * sig) @ q.T + centre
        chunks.append(pts)
    sh = np.concatenate(chunks, axis=0) if chunks else np.zeros((0, 3))
    if sh.shape[0] >= n_points:
        seg = sh[:n_points]
    else:
        noise = rng.random((n_points - sh.shape[0], 3)) * 10.0
        seg = np.concatenate([sh, noise], axis=0)
    rng.shuffle(seg, axis=0)
    return seg


def config3(n_per_segment: int = 100_000, n_segments: int = 10, k: int = 32,
            seed: int = 1003, grad_seed: int = 2003, n_showers: int = 200,
            mean_size: float = 450.0, with_grad: bool = True) -> Workload:
    """d=3, per segment `n_showers` anisotropic Gaussian showers (axis sigmas
    log-uniform in [0.01,0.5], random rotation, Poisson(mean_size) points) topped up
    with uniform noise to exactly n_per_segment points; forward + backward."""
    parts = [_shower_segment(_rng(seed + s), n_per_segment, n_showers, mean_size)
             for s in range(n_segments)]
    x = _f32(np.concatenate(parts, axis=0))
    n = x.shape[0]
    g = upstream_grad(n, k, grad_seed) if with_grad else None
    return Workload("C3_showers_d3", x, _splits([n_per_segment] * n_segments), k,
                    backward=True, grad_d2=g,
                    note="N=%d d=3 %d segments x %d showers + noise, k=%d"
                         % (n, n_segments, n_showers, k))


def config4(n: int = 500_000, k: int = 64, seed: int = 1004) -> Workload:
    """Single segment, d=8, uniform [-1,1); forward only; wide shells."""
    x = _rng(seed).random((n, 8)) * 2.0 - 1.0
    return Workload("C4_uniform_d8", _f32(x), _splits([n]), k,
                    note="N=%d d=8 U[-1,1) k=%d single segment" % (n, k))


def config5(n_per_segment: int = 1_000_000, n_segments: int = 5, k: int = 16,
            seed: int = 1005, grad_seed: int = 2005, n_hotspots: int = 1000,
            with_grad: bool = True) -> Workload:
    """d=2, strongly skewed density: 60 % of the points at radius U^3 with a uniform
    angle, 40 % in `n_hotspots` clusters of sigma 1e-3; forward + backward."""
    parts = []
    n_rad = (n_per_segment * 6) // 10
    n_hot = n_per_segment - n_rad
    for s in range(n_segments):
        rng = _rng(seed + s)
        r = rng.random(n_rad) ** 3
        th = rng.random(n_rad) * (2.0 * np.pi)
        rad = np.stack([r * np.cos(th), r * np.sin(th)], axis=1)
        centres = rng.random((n_hotspots, 2)) * 2.0 - 1.0
        which = np.arange(n_hot) % n_hotspots
        hot = centres[which] + 1e-3 * rng.standard_normal((n_hot, 2))
        seg = np.concatenate([rad, hot], axis=0)
        rng.shuffle(seg, axis=0)
        parts.append(seg)
    x = _f32(np.concatenate(parts, axis=0))
    n = x.shape[0]
    g = upstream_grad(n, k, grad_seed) if with_grad else None
    return Workload("C5_skewed_d2", x, _splits([n_per_segment] * n_segments), k,
                    backward=True, grad_d2=g,
                    note="N=%d d=2 r=U^3 + %d hotspots sigma=1e-3, %d segments, k=%d"
                         % (n, n_hotspots, n_segments, k))


def oc_association(sizes, objects_per_split: int, noise_frac: float, seed: int):
    """Synthetic object-condensation association (input of Algorithm 3, Section 5): every row split gets
    `objects_per_split` condensation points (vertices of the split); each other vertex is associated with one
    of them (skewed sizes) or, with probability noise_frac, with nothing (-1).  Returns asso_idx [n],
    unique_idx [n_unique], unique_rs_asso [n_unique], rs [S+1], n_maxuq, n_maxrs."""
    rng = _rng(seed)
    rs = _splits(sizes)
    asso = np.full(int(rs[-1]), -1, dtype=np.int32)
    uniq, uniq_rs = [], []
    for s, size in enumerate(sizes):
        if size == 0:
            continue
        b = int(rs[s])
        n_obj = min(objects_per_split, size)
        cps = np.sort(rng.choice(size, size=n_obj, replace=False)) + b
        weights = rng.random(n_obj) ** 3 + 1e-3
        pick = rng.choice(n_obj, size=size, p=weights / weights.sum())
        a = cps[pick].astype(np.int32)
        a[rng.random(size) < noise_frac] = -1
        a[cps - b] = cps                              # a condensation point belongs to itself
        asso[b:b + size] = a
        uniq += cps.tolist()
        uniq_rs += [s] * n_obj
    unique_idx = np.asarray(uniq, dtype=np.int32)
    unique_rs_asso = np.asarray(uniq_rs, dtype=np.int32)
    counts = np.bincount(asso[asso >= 0], minlength=1)
    n_maxuq = int(counts.max()) if counts.size else 1
    n_maxrs = int(max(sizes)) if len(sizes) else 1
    return asso, unique_idx, unique_rs_asso, rs, max(n_maxuq, 1), max(n_maxrs, 1)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


# --------------------------------------------------------------------------- #
# small structured / adversarial inputs for unit and parity tests
# --------------------------------------------------------------------------- #

def uniform(n: int, d: int, seed: int, lo: float = 0.0, hi: float = 1.0,
            sizes=None) -> tuple[np.ndarray, np.ndarray]:
    """n points uniform in [lo,hi)^d; `sizes` = per-segment sizes (default one segment)."""
    x = _rng(seed).random((n, d)) * (hi - lo) + lo
    if sizes is None:
        sizes = [n]
    assert sum(sizes) == n
    return _f32(x), _splits(sizes)


def lattice(m: int, d: int) -> tuple[np.ndarray, np.ndarray]:
    """Integer lattice {0..m-1}^d, row-major index order (last dim fastest)."""
    axes = np.meshgrid(*[np.arange(m)] * d, indexing="ij")
    x = np.stack([a.reshape(-1) for a in axes], axis=1)
    return _f32(x), _splits([x.shape[0]])


def collinear(n: int, d: int) -> tuple[np.ndarray, np.ndarray]:
    """x_i = (i, 0, ..., 0)."""
    x = np.zeros((n, d))
    x[:, 0] = np.arange(n)
    return _f32(x), _splits([n])


def duplicates(n: int, d: int, n_distinct: int, seed: int,
               sizes=None) -> tuple[np.ndarray, np.ndarray]:
    """n points drawn (with repetition) from n_distinct distinct locations."""
    rng = _rng(seed)
    base = rng.random((n_distinct, d))
    x = base[rng.integers(0, n_distinct, size=n)]
    if sizes is None:
        sizes = [n]
    return _f32(x), _splits(sizes)


def quantised(n: int, d: int, levels: int, seed: int,
              sizes=None) -> tuple[np.ndarray, np.ndarray]:
    """Coordinates on a coarse grid of `levels` values per dim: many exact d2 ties."""
    rng = _rng(seed)
    x = rng.integers(0, levels, size=(n, d)).astype(np.float64) / 8.0
    if sizes is None:
        sizes = [n]
    return _f32(x), _splits(sizes)


def ragged_sizes(n_segments: int, max_size: int, seed: int,
                 with_empty: bool = True) -> list[int]:
    """Random segment sizes in [0, max_size] (zeros included when with_empty)."""
    rng = _rng(seed)
    lo = 0 if with_empty else 1
    return [int(v) for v in rng.integers(lo, max_size + 1, size=n_segments)]
