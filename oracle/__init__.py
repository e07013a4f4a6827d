"""CPU oracle for the exact kNN graph build -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It shares no code with the HIP path and never imports it.

``knn`` / ``knn_rows`` / ``knn_backward`` wrap the plain C in ``knn_oracle.c`` (brute-force
definition of what Section 3 / Algorithm 2 of the paper computes, see that file's header).
``oc_helper`` wraps ``oc_helper_oracle.c`` (Algorithm 3).  ``paper_n_bins`` restates the bins-per-dimension heuristic of Section 3 (the displayed
equation and the clamp to [5, 30] stated under it).
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "knn_oracle.c")
_SRC_OC = os.path.join(_HERE, "oc_helper_oracle.c")
_LIB = os.path.join(_HERE, "libknn_oracle.so")
_lib = None

CFLAGS = ["-O3", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-std=gnu11", "-Wall"]


def build(force: bool = False) -> str:
    """Compile knn_oracle.c with gcc (no FMA contraction, no fast-math)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_OC))
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < newest
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, _SRC_OC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_knn.restype = ctypes.c_int
        lib.oracle_knn.argtypes = [f32p, i32p, i32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, i32p, f32p, ctypes.c_int]
        lib.oracle_knn_rows.restype = ctypes.c_int
        lib.oracle_knn_rows.argtypes = [f32p, i32p, i32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, i64p, ctypes.c_int64, i32p, f32p,
                                        ctypes.c_int]
        lib.oracle_knn_backward.restype = ctypes.c_int
        lib.oracle_knn_backward.argtypes = [f32p, i32p, f32p, ctypes.c_int64, ctypes.c_int,
                                            ctypes.c_int, f64p, f64p]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_oc_helper.restype = ctypes.c_int
        lib.oracle_oc_helper.argtypes = [i32p, i32p, i32p, i32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int64, i32p, i32p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _check_inputs(coords, row_splits):
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    row_splits = np.ascontiguousarray(row_splits, dtype=np.int32)
    assert coords.ndim == 2 and row_splits.ndim == 1 and row_splits.shape[0] >= 2
    assert row_splits[0] == 0 and row_splits[-1] == coords.shape[0]
    assert np.all(np.diff(row_splits) >= 0)
    return coords, row_splits


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dir_ptr(direction, n):
    if direction is None:
        return None, None
    direction = np.ascontiguousarray(direction, dtype=np.int32)
    assert direction.shape == (n,)
    return direction, _ptr(direction, ctypes.c_int32)


def knn(coords, row_splits, k: int, n_threads: int = 0, direction=None):
    """Exact kNN graph of every row: (idx int32 [n,k], d2 float32 [n,k]).
    direction: optional [n] flags of Algorithm 2 (0: neighbour only, 1: query only, 2: neither,
    anything else: both)."""
    coords, row_splits = _check_inputs(coords, row_splits)
    n, d = coords.shape
    direction, dptr = _dir_ptr(direction, n)
    idx = np.empty((n, k), dtype=np.int32)
    d2 = np.empty((n, k), dtype=np.float32)
    rc = _load().oracle_knn(_ptr(coords, ctypes.c_float), _ptr(row_splits, ctypes.c_int32), dptr,
                            n, d, row_splits.shape[0] - 1, k,
                            _ptr(idx, ctypes.c_int32), _ptr(d2, ctypes.c_float), n_threads)
    if rc != 0:
        raise ValueError("oracle_knn: bad arguments")
    return idx, d2


def knn_rows(coords, row_splits, k: int, rows, n_threads: int = 0, direction=None):
    """Exact kNN of the selected query rows only: ([len(rows),k], [len(rows),k])."""
    coords, row_splits = _check_inputs(coords, row_splits)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n, d = coords.shape
    direction, dptr = _dir_ptr(direction, n)
    idx = np.empty((rows.shape[0], k), dtype=np.int32)
    d2 = np.empty((rows.shape[0], k), dtype=np.float32)
    rc = _load().oracle_knn_rows(_ptr(coords, ctypes.c_float), _ptr(row_splits, ctypes.c_int32), dptr,
                                 n, d, row_splits.shape[0] - 1, k,
                                 _ptr(rows, ctypes.c_int64), rows.shape[0],
                                 _ptr(idx, ctypes.c_int32), _ptr(d2, ctypes.c_float), n_threads)
    if rc != 0:
        raise ValueError("oracle_knn_rows: bad arguments")
    return idx, d2


def knn_backward(grad_d2, idx, coords):
    """Analytic coordinate gradient in double: (grad [n,d] float64, abs_sum [n,d] float64)."""
    coords = np.ascontiguousarray(coords, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    grad_d2 = np.ascontiguousarray(grad_d2, dtype=np.float32)
    n, d = coords.shape
    k = idx.shape[1]
    assert idx.shape == grad_d2.shape == (n, k)
    g = np.empty((n, d), dtype=np.float64)
    a = np.empty((n, d), dtype=np.float64)
    rc = _load().oracle_knn_backward(_ptr(grad_d2, ctypes.c_float), _ptr(idx, ctypes.c_int32),
                                     _ptr(coords, ctypes.c_float), n, d, k,
                                     _ptr(g, ctypes.c_double), _ptr(a, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_knn_backward: bad arguments")
    return g, a


def oc_helper(asso_idx, unique_idx, unique_rs_asso, rs, n_maxuq: int, n_maxrs: int, calc_m_not: bool = True,
              rot_block: int = 1):
    """Index matrices of Algorithm 3 (Section 5).  Returns (M [n_maxuq, n_unique], M_not [n_maxrs, n_unique] or
    None): entry `fill` of object k is M[fill, k], the storage order of the paper's index macro."""
    asso_idx = np.ascontiguousarray(asso_idx, dtype=np.int32)
    unique_idx = np.ascontiguousarray(unique_idx, dtype=np.int32)
    unique_rs_asso = np.ascontiguousarray(unique_rs_asso, dtype=np.int32)
    rs = np.ascontiguousarray(rs, dtype=np.int32)
    n_unique = unique_idx.shape[0]
    M = np.empty((n_maxuq, n_unique), dtype=np.int32)
    M_not = np.empty((n_maxrs, n_unique), dtype=np.int32) if calc_m_not else None
    rc = _load().oracle_oc_helper(_ptr(asso_idx, ctypes.c_int32), _ptr(unique_idx, ctypes.c_int32),
                                  _ptr(unique_rs_asso, ctypes.c_int32), _ptr(rs, ctypes.c_int32),
                                  asso_idx.shape[0], n_unique, rs.shape[0] - 1, n_maxuq, n_maxrs,
                                  1 if calc_m_not else 0, rot_block, _ptr(M, ctypes.c_int32),
                                  _ptr(M_not, ctypes.c_int32) if calc_m_not else None)
    if rc != 0:
        raise ValueError("oracle_oc_helper: bad arguments")
    return M, M_not


def paper_n_bins(n_points: int, n_segments: int, k: int, d: int, d_max: int = 5):
    """Bins per dimension by the heuristic of Section 3:
    n_bins = (32 * n_elems / K) ** (1 / d_bin), n_elems the mean number of points per row
    split, d_bin = min(d, d_max) binning dimensions (Section 3, the paragraph on the limit of
    binning dimensions: at most the first 5), truncated to an integer and clamped to [5, 30].
    Returns (n_bins, d_bin)."""
    d_bin = min(d, d_max)
    n_elems = n_points / max(n_segments, 1)
    x = (32.0 * n_elems / k) ** (1.0 / d_bin) if n_elems > 0 else 0.0
    return max(5, min(30, int(math.floor(x)))), d_bin
