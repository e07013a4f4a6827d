"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (bins heuristic, workspace sizing, argument validation) behaves as the header says.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2511_10442_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fastgraph.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert B.status_string(0) == "FG_OK"
    for s in range(1, 6):
        assert B.status_string(s).startswith("FG_ERR_")
    assert "unknown" in B.status_string(99)


def test_auto_n_bins_paper_mode_matches_golden_and_oracle():
    for line in open(os.path.join(GOLDEN, "n_bins_paper.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        n, s, k, d = int(t[0]), int(t[1]), int(t[2]), int(t[3])
        assert B.fg_auto_n_bins(n, s, k, d, mode=0) == (int(t[5]), int(t[6]))
    for n in (10, 999, 12345, 10 ** 6):
        for s in (1, 3):
            for k in (1, 7, 40, 128):
                for d in range(2, 11):
                    assert B.fg_auto_n_bins(n, s, k, d, mode=0) == oracle.paper_n_bins(n, s, k, d)


def test_auto_n_bins_tuned_mode_is_sane():
    for n in (0, 1, 50, 4096, 10 ** 6, 5 * 10 ** 6):
        for s in (1, 10):
            for k in (1, 16, 128):
                for d in range(2, 11):
                    nb, db = B.fg_auto_n_bins(n, s, k, d, mode=1)
                    assert nb >= 1 and 2 <= db <= min(d, 5)
                    assert s * nb ** db <= (1 << 28)


def _status(fn, *args):
    return fn(*args)


def test_argument_validation_without_gpu():
    L = B.lib()
    nb, db = ctypes.c_int32(), ctypes.c_int32()
    sz = ctypes.c_size_t()
    assert L.fg_auto_n_bins(100, 1, 8, 3, 0, None, ctypes.byref(db)) == B.FG_ERR_NULL
    assert L.fg_auto_n_bins(100, 1, 8, 11, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_UNSUPPORTED
    assert L.fg_auto_n_bins(100, 1, 8, 1, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_UNSUPPORTED
    assert L.fg_auto_n_bins(100, 1, 129, 3, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_UNSUPPORTED
    assert L.fg_auto_n_bins(100, 0, 8, 3, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_auto_n_bins(-1, 1, 8, 3, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_auto_n_bins(1 << 31, 1, 8, 3, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_auto_n_bins(100, 1, 0, 3, 0, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_auto_n_bins(100, 1, 8, 3, 7, ctypes.byref(nb), ctypes.byref(db)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_workspace_size(100, 3, 1, 8, 0, 0, None) == B.FG_ERR_NULL
    assert L.fg_workspace_size(100, 3, 1, 8, 4, 6, ctypes.byref(sz)) == B.FG_ERR_UNSUPPORTED   # d_bin > 5
    assert L.fg_workspace_size(100, 3, 1, 8, 4, 4, ctypes.byref(sz)) == B.FG_ERR_UNSUPPORTED   # d_bin > d
    assert L.fg_workspace_size(100, 3, 1, 8, 4, 1, ctypes.byref(sz)) == B.FG_ERR_UNSUPPORTED   # d_bin < 2
    assert L.fg_workspace_size(100, 3, 1, 8, 2000, 3, ctypes.byref(sz)) == B.FG_ERR_BAD_SHAPE  # too many bins
    view = B._Binning()
    # errors are detected before anything is enqueued, so these are safe without a device
    assert L.fg_bin_points(None, None, 10, 3, 1, 4, 0, 0, None, 0, ctypes.byref(view), None) == B.FG_ERR_NULL
    assert L.fg_bin_points(8, 8, 10, 3, 1, 4, 0, 0, 256, 16, ctypes.byref(view), None) == B.FG_ERR_WORKSPACE
    assert L.fg_bin_points(8, 8, 10, 3, 1, 4, 0, 0, 257, 1 << 30, ctypes.byref(view), None) == B.FG_ERR_WORKSPACE
    assert L.fg_bin_points(8, 8, 10, 3, 1, 4, 0, 0, 256, 1 << 30, None, None) == B.FG_ERR_NULL
    assert L.fg_binned_select_knn(8, 8, 10, 3, 1, 4, 0, 0, None, 8, 256, 1 << 30, None) == B.FG_ERR_NULL
    assert L.fg_binned_select_knn(8, 8, 10, 12, 1, 4, 0, 0, 8, 8, 256, 1 << 30, None) == B.FG_ERR_UNSUPPORTED
    assert L.fg_binned_select_knn(None, None, 0, 3, 1, 4, 0, 0, None, None, None, 0, None) == B.FG_OK  # n == 0
    assert L.fg_knn_backward(None, 8, 8, None, 10, 3, 1, 4, 8, None, 0, None) == B.FG_ERR_NULL
    assert L.fg_knn_backward(8, 8, 8, None, 10, 3, 1, 200, 8, None, 0, None) == B.FG_ERR_UNSUPPORTED
    assert L.fg_knn_backward(8, 8, 8, 8, 10, 3, 1, 4, 8, 256, 16, None) == B.FG_ERR_WORKSPACE
    assert L.fg_knn_backward(None, None, None, None, 0, 3, 1, 4, None, None, 0, None) == B.FG_OK
    assert L.fg_query_binned(None, 8, 10, 3, 1, 4, 8, 8, None, None, None) == B.FG_ERR_NULL
    # the top of the advertised range: accepted up to FG_MAX_N = 2^31 - 2^16 points, refused beyond (the launch
    # arithmetic adds block sizes to n in 32 bits); likewise the number of row splits
    big = ctypes.c_size_t(0)
    assert L.fg_workspace_size(2147418112, 3, 1, 16, 0, 0, ctypes.byref(big)) == B.FG_OK and big.value > 2147418112 * 4 * 8
    for n_bad in (2147418113, 2 ** 31 - 1024, 2 ** 31 - 1, 2 ** 31, 2 ** 40):
        assert L.fg_workspace_size(n_bad, 3, 1, 16, 0, 0, ctypes.byref(big)) == B.FG_ERR_BAD_SHAPE
        assert L.fg_binned_select_knn(8, 8, n_bad, 3, 1, 16, 0, 0, 8, 8, 256, 1 << 40, None) == B.FG_ERR_BAD_SHAPE
        assert L.fg_knn_backward(8, 8, 8, None, n_bad, 3, 1, 16, 8, None, 0, None) == B.FG_ERR_BAD_SHAPE
    assert L.fg_workspace_size(10 ** 6, 3, (1 << 22) + 1, 16, 0, 0, ctypes.byref(big)) == B.FG_ERR_BAD_SHAPE
    assert L.fg_workspace_size(10 ** 7, 3, 1 << 22, 16, 2, 2, ctypes.byref(big)) == B.FG_OK
    assert L.fg_oc_helper(8, 8, 8, 8, 10, 2, 1, 4, 10, 1, 1, None, 8, None, 0, None) == B.FG_ERR_NULL
    assert L.fg_oc_helper(8, 8, 8, 8, 10, 2, 1, 4, 10, 1, 1, 8, None, None, 0, None) == B.FG_ERR_NULL
    assert L.fg_oc_helper(8, 8, 8, 8, 10, 2, 1, 0, 10, 0, 1, 8, None, None, 0, None) == B.FG_ERR_BAD_SHAPE
    assert L.fg_oc_helper(8, 8, 8, 8, 10, 2, 1, 4, 10, 0, 0, 8, None, None, 0, None) == B.FG_ERR_BAD_SHAPE
    assert L.fg_oc_helper(None, None, None, None, 10, 0, 1, 4, 10, 1, 1, None, None, None, 0, None) == B.FG_OK
    assert L.fg_oc_helper(8, 8, 8, 8, 10, 2, 1, 4, 10, 0, 1, 8, None, 256, 8, None) == B.FG_ERR_WORKSPACE
    assert B.fg_oc_helper_workspace_size(2000, 100000) >= (100000 // 128 + 1) * 2000 * 4


def test_workspace_size_scales_linearly():
    # (the size also covers the grid fg_knn_backward bins its rows with: a power of two near the automatic
    #  bin count, so compare sizes whose explicit grid is the larger of the two)
    a = B.fg_workspace_size(100_000, 3, 1, 16, 24, 3)
    b = B.fg_workspace_size(200_000, 3, 1, 16, 24, 3)
    # per point: bin_idx + rank + perm + work list + coordinates (d = 3 is given room for four) = 8 words,
    # plus two words per tile of 64 points for the tile order
    assert abs((b - a) - 100_000 * 4 * (8 + 2 / 64)) < 4096
    # per bin: one word for each of the four slices it is cut into along the last binning dimension (grids
    # well below the number of points; coarser cuts are chosen for larger ones)
    c = B.fg_workspace_size(100_000, 3, 1, 16, 34, 3)
    assert abs((c - a) - (34 ** 3 - 24 ** 3) * 4 * 4) < 8192
    # a table of four slices per bin would exceed twice the number of points: two slices
    e = B.fg_workspace_size(100_000, 3, 1, 16, 40, 3)
    assert abs((e - a) - (2 * 40 ** 3 - 4 * 24 ** 3) * 4) < 8192
    assert B.fg_workspace_size(0, 3, 1, 16) >= 0
