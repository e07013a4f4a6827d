"""Thin ctypes binding of libfastgraph_hip.so (same names as include/fastgraph.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI.
PyTorch is used for device memory and for the current HIP stream, nothing else.  There is no
CPU fallback: if the library has not been built this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastgraph_hip.so")

FG_OK = 0
FG_ERR_NULL = 1
FG_ERR_BAD_SHAPE = 2
FG_ERR_UNSUPPORTED = 3
FG_ERR_WORKSPACE = 4
FG_ERR_LAUNCH = 5

EXPORTS = ["fg_status_string", "fg_auto_n_bins", "fg_workspace_size", "fg_bin_points",
           "fg_binned_select_knn", "fg_binned_select_knn_static", "fg_binned_select_knn_dir", "fg_binned_select_knn_counted", "fg_query_binned",
           "fg_knn_backward", "fg_knn_backward_binned", "fg_oc_helper", "fg_oc_helper_workspace_size"]


class FgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s" % (where, status_string(status)))


class _Binning(ctypes.Structure):
    _fields_ = [("bin_idx", ctypes.c_void_p), ("bin_bounds", ctypes.c_void_p),
                ("sorted_points", ctypes.c_void_p), ("seg_geom", ctypes.c_void_p),
                ("cells_per_segment", ctypes.c_int64), ("n_bins", ctypes.c_int32),
                ("d_bin", ctypes.c_int32), ("sub_bins", ctypes.c_int32), ("record_floats", ctypes.c_int32),
                ("scratch", ctypes.c_void_p)]


class _QueryOptions(ctypes.Structure):
    _fields_ = [("dir", ctypes.c_void_p), ("algo", ctypes.c_int32), ("defer_lanes", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library; build it first if it is not there (never falls back to a CPU path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.fg_status_string.restype = ctypes.c_char_p
        L.fg_status_string.argtypes = [ctypes.c_int]
        L.fg_auto_n_bins.restype = ctypes.c_int
        L.fg_auto_n_bins.argtypes = [i64, i32, i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.fg_workspace_size.restype = ctypes.c_int
        L.fg_workspace_size.argtypes = [i64, i32, i32, i32, i32, i32, ctypes.POINTER(sz)]
        L.fg_bin_points.restype = ctypes.c_int
        L.fg_bin_points.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, sz,
                                    ctypes.POINTER(_Binning), vp]
        L.fg_binned_select_knn.restype = ctypes.c_int
        L.fg_binned_select_knn.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fg_binned_select_knn_static.restype = ctypes.c_int
        L.fg_binned_select_knn_static.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp]
        L.fg_binned_select_knn_dir.restype = ctypes.c_int
        L.fg_binned_select_knn_dir.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fg_binned_select_knn_counted.restype = ctypes.c_int
        L.fg_binned_select_knn_counted.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp,
                                                   vp, sz, vp]
        L.fg_query_binned.restype = ctypes.c_int
        L.fg_query_binned.argtypes = [ctypes.POINTER(_Binning), vp, i64, i32, i32, i32, vp, vp, vp,
                                      ctypes.POINTER(_QueryOptions), vp]
        L.fg_knn_backward.restype = ctypes.c_int
        L.fg_knn_backward.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, vp, vp, sz, vp]
        L.fg_knn_backward_binned.restype = ctypes.c_int
        L.fg_knn_backward_binned.argtypes = [ctypes.POINTER(_Binning), vp, vp, vp, i64, i32, i32, vp, vp]
        L.fg_oc_helper.restype = ctypes.c_int
        L.fg_oc_helper.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fg_oc_helper_workspace_size.restype = ctypes.c_int
        L.fg_oc_helper_workspace_size.argtypes = [i64, i32, ctypes.POINTER(sz)]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fg_status_string(int(status)).decode()


fg_status_string = status_string


def _check(status: int, where: str):
    if status != FG_OK:
        raise FgError(status, where)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError("%s must be contiguous %s" % (name, dtype))
    return t


def _ptr(t) -> int:
    return 0 if t is None or t.numel() == 0 else int(t.data_ptr())


def fg_auto_n_bins(n: int, n_segments: int, k: int, d: int, mode: int = 1):
    nb, db = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().fg_auto_n_bins(n, n_segments, k, d, mode, ctypes.byref(nb), ctypes.byref(db)),
           "fg_auto_n_bins")
    return int(nb.value), int(db.value)


def fg_workspace_size(n: int, d: int, n_segments: int, k: int, n_bins: int = 0, d_bin: int = 0) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().fg_workspace_size(n, d, n_segments, k, n_bins, d_bin, ctypes.byref(out)),
           "fg_workspace_size")
    return int(out.value)


def alloc_workspace(n: int, d: int, n_segments: int, k: int, n_bins: int = 0, d_bin: int = 0,
                    device="cuda") -> torch.Tensor:
    size = fg_workspace_size(n, d, n_segments, k, n_bins, d_bin)
    return torch.empty(max(size, 256), dtype=torch.uint8, device=device)


@dataclass
class Binning:
    """Views into the workspace (kept alive here) produced by fg_bin_points."""
    raw: _Binning
    workspace: torch.Tensor
    n: int
    d: int
    n_segments: int
    n_bins: int
    d_bin: int
    cells_per_segment: int
    record_floats: int
    sub_bins: int

    def _view(self, ptr: int, count: int, dtype) -> torch.Tensor:
        off = ptr - self.workspace.data_ptr()
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return self.workspace[off:off + nbytes].view(dtype)

    @property
    def bin_idx(self):
        return self._view(self.raw.bin_idx, self.n, torch.int32)

    @property
    def sorted_records(self):
        """[n, record_floats] float32: coordinates, original row index (int32 bits), zero padding."""
        return self._view(self.raw.sorted_points, self.n * self.record_floats, torch.float32).view(self.n, self.record_floats)

    @property
    def perm(self):
        """Sorted position -> original row: the index field of the records."""
        return self.sorted_records.view(torch.int32)[:, self.d].contiguous()

    @property
    def sorted_coords(self):
        """[n, d] coordinates in bin order."""
        return self.sorted_records[:, :self.d]

    @property
    def bin_bounds(self):
        return self._view(self.raw.bin_bounds, self.n_segments * self.cells_per_segment + 1, torch.int32)

    @property
    def work_count(self):
        """Number of queries the tile kernel handed to the list kernel in the last query call (the one word of
        the scratch block that the header documents)."""
        return self._view(self.raw.scratch, 1, torch.int32)

    @property
    def seg_geom(self):
        return self._view(self.raw.seg_geom, self.n_segments * self.d_bin * 4, torch.float32).view(
            self.n_segments, self.d_bin, 4)


def fg_bin_points(coords: torch.Tensor, row_splits: torch.Tensor, k_hint: int, n_bins: int = 0,
                  d_bin: int = 0, workspace: torch.Tensor | None = None) -> Binning:
    coords = _dev(coords, torch.float32, "coords")
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    n, d = coords.shape
    s = row_splits.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(n, d, s, k_hint, n_bins, d_bin, coords.device)
    raw = _Binning()
    _check(lib().fg_bin_points(_ptr(coords), _ptr(row_splits), n, d, s, k_hint, n_bins, d_bin,
                               _ptr(workspace), workspace.numel(), ctypes.byref(raw), _stream()),
           "fg_bin_points")
    return Binning(raw, workspace, n, d, s, int(raw.n_bins), int(raw.d_bin),
                   int(raw.cells_per_segment), int(raw.record_floats), int(raw.sub_bins))


def _out(t, shape, dtype, device, name: str) -> torch.Tensor:
    """A caller-supplied output tensor must be exactly what the kernels write: device, dtype, shape, contiguous."""
    if t is None:
        return torch.empty(shape, dtype=dtype, device=device)
    _dev(t, dtype, name)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t


def fg_query_binned(binning: Binning, row_splits: torch.Tensor, k: int, out_idx=None, out_d2=None,
                    out_candidates=None, direction: torch.Tensor | None = None, algo: int = 0,
                    defer_lanes: int = -1):
    """direction, algo, defer_lanes: the fields of fg_query_options (None / 0 / -1 = defaults)."""
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    n = binning.n
    dev = binning.workspace.device
    out_idx = _out(out_idx, (n, k), torch.int32, dev, "out_idx")
    out_d2 = _out(out_d2, (n, k), torch.float32, dev, "out_d2")
    if out_candidates is not None:
        _out(out_candidates, (n,), torch.int32, dev, "out_candidates")
    opt = _QueryOptions()
    if direction is not None:
        direction = _dev(direction, torch.int32, "direction")
        if direction.numel() != n:
            raise ValueError("direction must have one flag per point")
    opt.dir = _ptr(direction) or None
    opt.algo = algo
    opt.defer_lanes = defer_lanes
    _check(lib().fg_query_binned(ctypes.byref(binning.raw), _ptr(row_splits), n, binning.d,
                                 binning.n_segments, k, _ptr(out_idx), _ptr(out_d2),
                                 _ptr(out_candidates), ctypes.byref(opt), _stream()), "fg_query_binned")
    return out_idx, out_d2


def fg_binned_select_knn(coords: torch.Tensor, row_splits: torch.Tensor, k: int, n_bins: int = 0,
                         d_bin: int = 0, workspace: torch.Tensor | None = None, out_idx=None,
                         out_d2=None):
    coords = _dev(coords, torch.float32, "coords")
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    n, d = coords.shape
    s = row_splits.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(n, d, s, k, n_bins, d_bin, coords.device)
    out_idx = _out(out_idx, (n, k), torch.int32, coords.device, "out_idx")
    out_d2 = _out(out_d2, (n, k), torch.float32, coords.device, "out_d2")
    _check(lib().fg_binned_select_knn(_ptr(coords), _ptr(row_splits), n, d, s, k, n_bins, d_bin,
                                      _ptr(out_idx), _ptr(out_d2), _ptr(workspace),
                                      workspace.numel(), _stream()), "fg_binned_select_knn")
    return out_idx, out_d2


FG_STATIC_SCRATCH_BYTES = 32 << 20


def fg_binned_select_knn_static(coords: torch.Tensor, row_splits: torch.Tensor, k: int, out_idx: torch.Tensor,
                                out_d2: torch.Tensor, n_bins: int = 0, d_bin: int = 0):
    """The entry point that allocates nothing: the caller passes inputs and outputs, the scratch is the library's
    own device array.  (The binding allocates nothing either: both outputs are required.)"""
    coords = _dev(coords, torch.float32, "coords")
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    n, d = coords.shape
    s = row_splits.numel() - 1
    _out(out_idx, (n, k), torch.int32, coords.device, "out_idx")
    _out(out_d2, (n, k), torch.float32, coords.device, "out_d2")
    _check(lib().fg_binned_select_knn_static(_ptr(coords), _ptr(row_splits), n, d, s, k, n_bins, d_bin,
                                             _ptr(out_idx), _ptr(out_d2), _stream()),
           "fg_binned_select_knn_static")
    return out_idx, out_d2


def fg_binned_select_knn_dir(coords: torch.Tensor, row_splits: torch.Tensor, direction: torch.Tensor, k: int,
                             n_bins: int = 0, d_bin: int = 0, workspace: torch.Tensor | None = None,
                             out_idx=None, out_d2=None):
    """Direction-flag variant: direction [n] int32 (0 neighbour only, 1 query only, 2 neither, else both)."""
    coords = _dev(coords, torch.float32, "coords")
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    direction = _dev(direction, torch.int32, "direction")
    n, d = coords.shape
    if direction.numel() != n:
        raise ValueError("direction must have one flag per point")
    s = row_splits.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(n, d, s, k, n_bins, d_bin, coords.device)
    out_idx = _out(out_idx, (n, k), torch.int32, coords.device, "out_idx")
    out_d2 = _out(out_d2, (n, k), torch.float32, coords.device, "out_d2")
    _check(lib().fg_binned_select_knn_dir(_ptr(coords), _ptr(row_splits), _ptr(direction), n, d, s, k, n_bins,
                                          d_bin, _ptr(out_idx), _ptr(out_d2), _ptr(workspace),
                                          workspace.numel(), _stream()), "fg_binned_select_knn_dir")
    return out_idx, out_d2


def fg_binned_select_knn_counted(coords: torch.Tensor, row_splits: torch.Tensor, k: int,
                                 n_bins: int = 0, d_bin: int = 0,
                                 workspace: torch.Tensor | None = None):
    coords = _dev(coords, torch.float32, "coords")
    row_splits = _dev(row_splits, torch.int32, "row_splits")
    n, d = coords.shape
    s = row_splits.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(n, d, s, k, n_bins, d_bin, coords.device)
    out_idx = torch.empty((n, k), dtype=torch.int32, device=coords.device)
    out_d2 = torch.empty((n, k), dtype=torch.float32, device=coords.device)
    cand = torch.empty((n,), dtype=torch.int32, device=coords.device)
    _check(lib().fg_binned_select_knn_counted(_ptr(coords), _ptr(row_splits), n, d, s, k, n_bins,
                                              d_bin, _ptr(out_idx), _ptr(out_d2), _ptr(cand),
                                              _ptr(workspace), workspace.numel(), _stream()),
           "fg_binned_select_knn_counted")
    return out_idx, out_d2, cand


def fg_knn_backward(grad_d2: torch.Tensor, idx: torch.Tensor, coords: torch.Tensor,
                    row_splits: torch.Tensor | None = None, grad_coords: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None) -> torch.Tensor:
    """With row_splits the bin-ordered LDS-combining kernel runs (a workspace is allocated if none
    is passed); without, the plain atomic scatter."""
    grad_d2 = _dev(grad_d2, torch.float32, "grad_d2")
    idx = _dev(idx, torch.int32, "idx")
    coords = _dev(coords, torch.float32, "coords")
    n, d = coords.shape
    k = idx.shape[1]
    if tuple(grad_d2.shape) != (n, k) or idx.shape[0] != n:
        raise ValueError("grad_d2 and idx must be [n, k]")
    grad_coords = _out(grad_coords, (n, d), torch.float32, coords.device, "grad_coords")
    s = 0
    if row_splits is not None:
        row_splits = _dev(row_splits, torch.int32, "row_splits")
        s = row_splits.numel() - 1
        if workspace is None:
            workspace = alloc_workspace(n, d, s, k, 0, 0, coords.device)
    else:
        workspace = None
    _check(lib().fg_knn_backward(_ptr(grad_d2), _ptr(idx), _ptr(coords), _ptr(row_splits), n, d, s, k,
                                 _ptr(grad_coords), _ptr(workspace),
                                 0 if workspace is None else workspace.numel(), _stream()), "fg_knn_backward")
    return grad_coords


def fg_knn_backward_binned(binning: Binning, grad_d2: torch.Tensor, idx: torch.Tensor, coords: torch.Tensor,
                           grad_coords: torch.Tensor | None = None) -> torch.Tensor:
    """Backward on the binning the forward used (fg_bin_points on the same coords, workspace untouched since)."""
    grad_d2 = _dev(grad_d2, torch.float32, "grad_d2")
    idx = _dev(idx, torch.int32, "idx")
    coords = _dev(coords, torch.float32, "coords")
    n, d = coords.shape
    k = idx.shape[1]
    if tuple(grad_d2.shape) != (n, k) or idx.shape[0] != n or n != binning.n or d != binning.d:
        raise ValueError("grad_d2 and idx must be [n, k] for the binned coords [n, d]")
    grad_coords = _out(grad_coords, (n, d), torch.float32, coords.device, "grad_coords")
    _check(lib().fg_knn_backward_binned(ctypes.byref(binning.raw), _ptr(grad_d2), _ptr(idx), _ptr(coords), n, d, k,
                                        _ptr(grad_coords), _stream()), "fg_knn_backward_binned")
    return grad_coords


def fg_oc_helper_workspace_size(n_unique: int, n_maxrs: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().fg_oc_helper_workspace_size(n_unique, n_maxrs, ctypes.byref(out)), "fg_oc_helper_workspace_size")
    return int(out.value)


def fg_oc_helper(asso_idx: torch.Tensor, unique_idx: torch.Tensor, unique_rs_asso: torch.Tensor, rs: torch.Tensor,
                 n_maxuq: int, n_maxrs: int, calc_m_not: bool = True, rot_block: int = 1, M=None, M_not=None,
                 workspace="auto"):
    """Index matrices of Algorithm 3: returns (M [n_maxuq, n_unique], M_not [n_maxrs, n_unique] or None).
    workspace: "auto" allocates the scratch of the chunked kernels, None runs the single-kernel form."""
    asso_idx = _dev(asso_idx, torch.int32, "asso_idx")
    unique_idx = _dev(unique_idx, torch.int32, "unique_idx")
    unique_rs_asso = _dev(unique_rs_asso, torch.int32, "unique_rs_asso")
    rs = _dev(rs, torch.int32, "rs")
    n_unique = unique_idx.numel()
    if M is None:
        M = torch.empty((n_maxuq, n_unique), dtype=torch.int32, device=asso_idx.device)
    if calc_m_not and M_not is None:
        M_not = torch.empty((n_maxrs, n_unique), dtype=torch.int32, device=asso_idx.device)
    if isinstance(workspace, str):
        workspace = torch.empty(max(256, fg_oc_helper_workspace_size(n_unique, n_maxrs)), dtype=torch.uint8,
                                device=asso_idx.device)
    _check(lib().fg_oc_helper(_ptr(asso_idx), _ptr(unique_idx), _ptr(unique_rs_asso), _ptr(rs), asso_idx.numel(),
                              n_unique, rs.numel() - 1, n_maxuq, n_maxrs, 1 if calc_m_not else 0, rot_block,
                              _ptr(M), _ptr(M_not) if calc_m_not else 0, _ptr(workspace),
                              0 if workspace is None else workspace.numel(), _stream()), "fg_oc_helper")
    return M, (M_not if calc_m_not else None)
