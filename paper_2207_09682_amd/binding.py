"""Thin ctypes binding over libqgbdt.so (see include/qgbdt.h).

Argument marshalling only: every step runs in the library's HIP kernels.  torch
is used for device memory and the current stream.  There is no CPU path: the
import of the library and every call fail loudly when the HIP library or a GPU
is missing.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libqgbdt.so")

ROUND_STOCHASTIC = 0
ROUND_NEAREST = 1
ROWS_AUTO, ROWS_IDS, ROWS_IDS_GH, ROWS_ORDERED = 0, 1, 2, 3
WS_BIND, WS_ROW_COPIES, WS_BOOST = 1, 2, 4
E_WORKSPACE = -6

EXPORTS = [
    "qgbdt_create", "qgbdt_destroy", "qgbdt_set_stream", "qgbdt_last_error", "qgbdt_workspace_bytes",
    "qgbdt_set_workspace",
    "qgbdt_quantize_gradients", "qgbdt_build_histograms", "qgbdt_subtract_histograms",
    "qgbdt_find_best_splits", "qgbdt_find_best_splits_static", "qgbdt_partition_rows", "qgbdt_refit_leaves", "qgbdt_grow_tree",
    "qgbdt_logistic_gradients", "qgbdt_lambdarank_gradients", "qgbdt_update_scores", "qgbdt_boost_iteration",
    "qgbdt_boost_iteration_lambdarank",
    "qgbdt_set_profiling", "qgbdt_read_profile", "qgbdt_read_profile_roots", "qgbdt_tree_stats", "qgbdt_bind_bins",
    "qgbdt_measure_stream_read", "qgbdt_describe_hist_plan",
]


class Shape(C.Structure):
    _fields_ = [("n_rows", C.c_int64), ("n_features", C.c_int32), ("n_bins", C.c_int32),
                ("bin_bytes", C.c_int32), ("max_leaves", C.c_int32)]


class Params(C.Structure):
    _fields_ = [("bits_g", C.c_int32), ("bits_h", C.c_int32), ("rounding", C.c_int32),
                ("num_leaves", C.c_int32), ("min_data_in_leaf", C.c_int32), ("acc_width", C.c_int32),
                ("row_layout", C.c_int32), ("seed", C.c_uint64), ("min_sum_hessian", C.c_double)]


class TreePtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "n_leaves", "split_leaf", "split_feature", "split_bin", "split_gain", "split_stats",
        "split_n_left", "leaf_begin", "leaf_count", "leaf_sum_g", "leaf_sum_h", "leaf_value",
        "leaf_value_quant", "delta", "hist_units")]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2207_09682_amd.build` "
                               "(there is no CPU fallback)")
        lib = C.CDLL(LIB_PATH)
        lib.qgbdt_last_error.restype = C.c_char_p
        lib.qgbdt_last_error.argtypes = [C.c_void_p]
        lib.qgbdt_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Shape), C.c_void_p]
        lib.qgbdt_destroy.argtypes = [C.c_void_p]
        lib.qgbdt_set_stream.argtypes = [C.c_void_p, C.c_void_p]
        lib.qgbdt_workspace_bytes.argtypes = [C.POINTER(Shape), C.c_uint32, C.POINTER(C.c_size_t)]
        lib.qgbdt_set_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_uint32]
        lib.qgbdt_quantize_gradients.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                                 C.c_uint64, C.c_uint32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.qgbdt_build_histograms.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                               C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        lib.qgbdt_subtract_histograms.argtypes = [C.c_void_p] * 4
        lib.qgbdt_find_best_splits.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                               C.c_double, C.c_void_p]
        lib.qgbdt_find_best_splits_static.argtypes = lib.qgbdt_find_best_splits.argtypes
        lib.qgbdt_partition_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int32,
                                             C.c_int32, C.c_void_p]
        lib.qgbdt_refit_leaves.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int32, C.c_void_p]
        lib.qgbdt_grow_tree.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params), C.c_uint32,
                                        C.POINTER(TreePtrs), C.c_void_p]
        lib.qgbdt_logistic_gradients.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.qgbdt_lambdarank_gradients.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                                   C.c_void_p]
        lib.qgbdt_boost_iteration_lambdarank.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                                         C.POINTER(Params), C.c_uint32, C.c_double,
                                                         C.POINTER(TreePtrs), C.c_void_p]
        lib.qgbdt_update_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int32, C.c_double]
        lib.qgbdt_boost_iteration.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params),
                                              C.c_uint32, C.c_double, C.POINTER(TreePtrs), C.c_void_p]
        lib.qgbdt_set_profiling.argtypes = [C.c_void_p, C.c_int32]
        lib.qgbdt_read_profile.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        lib.qgbdt_read_profile_roots.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        lib.qgbdt_tree_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        lib.qgbdt_bind_bins.argtypes = [C.c_void_p, C.c_void_p]
        lib.qgbdt_measure_stream_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_double),
                                                  C.POINTER(C.c_int32)]
        lib.qgbdt_describe_hist_plan.argtypes = [C.POINTER(Shape), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                                 C.c_int32, C.POINTER(C.c_int64), C.c_int32]
        _lib = lib
    return _lib


PLAN_FIELDS = ("ft", "ftp", "dpr", "rows_per_it", "n_tiles", "threads", "lds_bytes", "chunk_rows", "max_groups",
               "max_lanes", "min_rows_per_group", "acc_width", "hshift", "flat_lanes", "flat_rows", "max_items",
               "slot_bytes", "single_rows", "pad16", "wide_v", "ragged", "bytewise", "target_rows", "partial_bytes",
               "two_level")


def describe_hist_plan(n_rows, n_features, n_bins, max_leaves=255, bin_bytes=1, bits_g=3, bits_h=3, acc_width=0,
                       skewed=False, rows=0, n_builds=1) -> dict:
    """qgbdt_describe_hist_plan: the histogram launch plan of a shape as a dict (host-only, needs no GPU)."""
    lib = load_library()
    shape = Shape(n_rows, n_features, n_bins, bin_bytes, max_leaves)
    out = (C.c_int64 * 25)()
    rc = lib.qgbdt_describe_hist_plan(C.byref(shape), bits_g, bits_h, acc_width, 1 if skewed else 0, rows, n_builds, out, 25)
    if rc != 0:
        raise QgbdtError(rc, lib.qgbdt_last_error(None).decode())
    return dict(zip(PLAN_FIELDS, (int(x) for x in out)))


class QgbdtError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"qgbdt error {code}: {msg}")
        self.code = code


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


@dataclass
class Tree:
    """Device tensors written by grow_tree (see qgbdt_tree in include/qgbdt.h)."""
    n_leaves: torch.Tensor
    split_leaf: torch.Tensor
    split_feature: torch.Tensor
    split_bin: torch.Tensor
    split_gain: torch.Tensor
    split_stats: torch.Tensor
    split_n_left: torch.Tensor
    leaf_begin: torch.Tensor
    leaf_count: torch.Tensor
    leaf_sum_g: torch.Tensor
    leaf_sum_h: torch.Tensor
    leaf_value: torch.Tensor
    leaf_value_quant: torch.Tensor
    delta: torch.Tensor
    hist_units: torch.Tensor
    row_idx: torch.Tensor

    def ptrs(self) -> TreePtrs:
        p = TreePtrs()
        for name, _ in TreePtrs._fields_:
            setattr(p, name, getattr(self, name).data_ptr())
        return p


class Context:
    """One qgbdt context: a problem shape, its device workspace (one torch tensor, owned here) and a stream.

    `workspace_flags` names the optional sections of the workspace (WS_BIND: bind_bins, WS_ROW_COPIES: leaf-ordered
    copies of narrow rows, WS_BOOST: boost_iteration); the default asks for all of them."""

    def __init__(self, n_rows: int, n_features: int, n_bins: int, max_leaves: int = 255, bin_bytes: int = 1,
                 device: str | torch.device = "cuda:0", workspace_flags: int = WS_BIND | WS_ROW_COPIES | WS_BOOST):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the qgbdt library runs on MI355X only (no CPU path)")
        self.lib = load_library()
        self.device = torch.device(device)
        self.shape = Shape(n_rows, n_features, n_bins, bin_bytes, max_leaves)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            rc = self.lib.qgbdt_create(C.byref(self._h), C.byref(self.shape), C.c_void_p(stream))
        if rc != 0:
            raise QgbdtError(rc, self.lib.qgbdt_last_error(None).decode())
        self.workspace = None
        self.set_workspace(flags=workspace_flags)

    @staticmethod
    def workspace_bytes_for(n_rows: int, n_features: int, n_bins: int, max_leaves: int = 255, bin_bytes: int = 1,
                            flags: int = WS_BIND | WS_ROW_COPIES | WS_BOOST) -> int:
        """qgbdt_workspace_bytes: device bytes a context of this shape needs (no context, no GPU call)."""
        lib = load_library()
        shape = Shape(n_rows, n_features, n_bins, bin_bytes, max_leaves)
        n = C.c_size_t(0)
        rc = lib.qgbdt_workspace_bytes(C.byref(shape), flags, C.byref(n))
        if rc != 0:
            raise QgbdtError(rc, lib.qgbdt_last_error(None).decode())
        return n.value

    def set_workspace(self, workspace: torch.Tensor | None = None, flags: int = WS_BIND | WS_ROW_COPIES | WS_BOOST):
        """qgbdt_set_workspace with `workspace` (a contiguous uint8 device tensor, 256-byte aligned) or, when None,
        with a tensor of exactly the needed size allocated here.  The tensor is kept alive by the context."""
        if workspace is None:
            s = self.shape
            need = self.workspace_bytes_for(s.n_rows, s.n_features, s.n_bins, s.max_leaves, s.bin_bytes, flags)
            workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        self._sync_stream()
        self._chk(self.lib.qgbdt_set_workspace(self._h, C.c_void_p(_dev(workspace, torch.uint8, "workspace")),
                                               workspace.numel(), flags))
        self.workspace = workspace
        self.workspace_flags = flags

    def detach_workspace(self):
        """qgbdt_set_workspace(NULL): the context gives its block back; every step but the ones that need no
        workspace refuses until another block is set."""
        self._sync_stream()
        self._chk(self.lib.qgbdt_set_workspace(self._h, None, 0, 0))
        self.workspace = None
        self.workspace_flags = 0

    def bind_bins(self, bins: torch.Tensor | None) -> None:
        """qgbdt_bind_bins: keep a feature-major copy of `bins` for the partitions of the trees that follow
        (None forgets it).  The tensor must stay alive and unchanged while it is bound."""
        self._chk(self.lib.qgbdt_bind_bins(self._h, C.c_void_p(self._bins(bins)) if bins is not None else None))

    # -- helpers ---------------------------------------------------------------
    def _bins(self, bins: torch.Tensor) -> int:
        """Device pointer of the bin matrix: uint8, or uint16 for a context created with bin_bytes=2."""
        return _dev(bins, torch.uint16 if self.shape.bin_bytes == 2 else torch.uint8, "bins")

    def _chk(self, rc: int):
        if rc != 0:
            raise QgbdtError(rc, self.lib.qgbdt_last_error(self._h).decode())

    def _sync_stream(self):
        self.lib.qgbdt_set_stream(self._h, C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream))

    def close(self):
        if self._h:
            self.lib.qgbdt_destroy(self._h)   # synchronises the stream: the workspace may be released afterwards
            self._h = C.c_void_p()
        self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self) -> int:
        """Bytes of the workspace tensor this context holds."""
        return 0 if self.workspace is None else self.workspace.numel()

    # -- steps -------------------------------------------------------------------
    def quantize_gradients(self, g, h, bits_g, bits_h, seed, iteration, rounding=ROUND_STOCHASTIC, gh_out=None,
                           delta_out=None):
        self._sync_stream()
        n = g.numel()
        gh = gh_out if gh_out is not None else torch.empty(n, dtype=torch.int16, device=self.device)
        delta = delta_out if delta_out is not None else torch.empty(2, dtype=torch.float32, device=self.device)
        self._chk(self.lib.qgbdt_quantize_gradients(self._h, _dev(g, torch.float32, "g"), _dev(h, torch.float32, "h"),
                                                    n, bits_g, bits_h, seed, iteration, rounding,
                                                    _dev(gh, torch.int16, "gh_out"), _dev(delta, torch.float32, "delta_out")))
        return gh, delta

    def build_histograms(self, bins, gh, row_idx=None, begin=0, count=None, bits_g=3, bits_h=3, acc_width=0,
                         hist_out=None):
        self._sync_stream()
        if count is None:
            count = (row_idx.numel() if row_idx is not None else bins.shape[0]) - begin
        W = self.shape.n_features * self.shape.n_bins
        hist = hist_out if hist_out is not None else torch.empty(W, dtype=torch.int64, device=self.device)
        self._chk(self.lib.qgbdt_build_histograms(
            self._h, self._bins(bins), _dev(gh, torch.int16, "gh"),
            _dev(row_idx, torch.int32, "row_idx") if row_idx is not None else None, begin, count, bits_g, bits_h,
            acc_width, _dev(hist, torch.int64, "hist_out")))
        return hist

    def subtract_histograms(self, parent, child, out=None):
        self._sync_stream()
        out = out if out is not None else torch.empty_like(parent)
        self._chk(self.lib.qgbdt_subtract_histograms(self._h, _dev(parent, torch.int64, "parent"),
                                                     _dev(child, torch.int64, "child"), _dev(out, torch.int64, "out")))
        return out

    def find_best_splits(self, hist, stats, delta, min_data_in_leaf=20, min_sum_hessian=0.0):
        """hist: int64 [n, nb*F] (bin-major); stats: int64 [n, 3] (n_rows, sum_g, sum_h).
        Returns a uint8 tensor [n, 56] holding qgbdt_split records (see unpack_splits)."""
        self._sync_stream()
        n = stats.shape[0]
        out = torch.empty((n, 56), dtype=torch.uint8, device=self.device)
        self._chk(self.lib.qgbdt_find_best_splits(self._h, _dev(hist, torch.int64, "hist"), n,
                                                  _dev(stats, torch.int64, "stats"), _dev(delta, torch.float32, "delta"),
                                                  min_data_in_leaf, min_sum_hessian, out.data_ptr()))
        return out

    def find_best_splits_static(self, hist, stats, delta, out, min_data_in_leaf=20, min_sum_hessian=0.0):
        """qgbdt_find_best_splits_static: the same search with the library's fixed scratch; allocates nothing, so
        the caller passes `out` (uint8 [n, 56])."""
        self._sync_stream()
        n = stats.shape[0]
        self._chk(self.lib.qgbdt_find_best_splits_static(self._h, _dev(hist, torch.int64, "hist"), n,
                                                         _dev(stats, torch.int64, "stats"),
                                                         _dev(delta, torch.float32, "delta"), min_data_in_leaf,
                                                         min_sum_hessian, _dev(out, torch.uint8, "out")))
        return out

    def partition_rows(self, bins, row_idx, begin, count, feature, bin):
        self._sync_stream()
        n_left = torch.empty(1, dtype=torch.int64, device=self.device)
        self._chk(self.lib.qgbdt_partition_rows(self._h, self._bins(bins),
                                                _dev(row_idx, torch.int32, "row_idx"), begin, count, feature, bin,
                                                n_left.data_ptr()))
        return n_left

    def refit_leaves(self, g, h, row_idx, leaf_begin, leaf_count):
        self._sync_stream()
        n = leaf_begin.numel()
        out = torch.empty(n, dtype=torch.float64, device=self.device)
        self._chk(self.lib.qgbdt_refit_leaves(self._h, _dev(g, torch.float32, "g"), _dev(h, torch.float32, "h"),
                                              _dev(row_idx, torch.int32, "row_idx"),
                                              _dev(leaf_begin, torch.int64, "leaf_begin"),
                                              _dev(leaf_count, torch.int64, "leaf_count"), n, out.data_ptr()))
        return out

    def new_tree(self) -> Tree:
        L = self.shape.max_leaves
        S = max(L - 1, 1)
        d = self.device
        z = lambda n, dt: torch.zeros(n, dtype=dt, device=d)
        return Tree(z(1, torch.int32), z(S, torch.int32), z(S, torch.int32), z(S, torch.int32), z(S, torch.float64),
                    z(S * 4, torch.int64), z(S, torch.int64), z(L, torch.int64), z(L, torch.int64), z(L, torch.int64),
                    z(L, torch.int64), z(L, torch.float64), z(L, torch.float64), z(2, torch.float32),
                    z(1, torch.int64), z(self.shape.n_rows, torch.int32))

    def grow_tree(self, bins, g, h, bits_g, bits_h, seed, iteration, num_leaves, min_data_in_leaf=20,
                  min_sum_hessian=0.0, rounding=ROUND_STOCHASTIC, acc_width=0, tree: Tree | None = None,
                  row_layout=ROWS_AUTO) -> Tree:
        self._sync_stream()
        tree = tree if tree is not None else self.new_tree()
        p = Params(bits_g, bits_h, rounding, num_leaves, min_data_in_leaf, acc_width, row_layout, seed, min_sum_hessian)
        tp = tree.ptrs()
        self._chk(self.lib.qgbdt_grow_tree(self._h, self._bins(bins), _dev(g, torch.float32, "g"),
                                           _dev(h, torch.float32, "h"), C.byref(p), iteration, C.byref(tp),
                                           _dev(tree.row_idx, torch.int32, "row_idx")))
        return tree

    # -- around the tree ---------------------------------------------------------
    def logistic_gradients(self, score, label):
        self._sync_stream()
        n = score.numel()
        g = torch.empty(n, dtype=torch.float32, device=self.device)
        h = torch.empty(n, dtype=torch.float32, device=self.device)
        self._chk(self.lib.qgbdt_logistic_gradients(self._h, _dev(score, torch.float32, "score"),
                                                    _dev(label, torch.float32, "label"), n, g.data_ptr(), h.data_ptr()))
        return g, h

    def lambdarank_gradients(self, score, relevance, group_size):
        self._sync_stream()
        n = score.numel()
        g = torch.empty(n, dtype=torch.float32, device=self.device)
        h = torch.empty(n, dtype=torch.float32, device=self.device)
        self._chk(self.lib.qgbdt_lambdarank_gradients(self._h, _dev(score, torch.float32, "score"),
                                                      _dev(relevance, torch.float32, "relevance"), n, int(group_size),
                                                      g.data_ptr(), h.data_ptr()))
        return g, h

    def update_scores(self, score, row_idx, leaf_begin, leaf_count, leaf_value, learning_rate):
        """Updates `score` in place."""
        self._sync_stream()
        self._chk(self.lib.qgbdt_update_scores(self._h, _dev(score, torch.float32, "score"),
                                               _dev(row_idx, torch.int32, "row_idx"),
                                               _dev(leaf_begin, torch.int64, "leaf_begin"),
                                               _dev(leaf_count, torch.int64, "leaf_count"),
                                               _dev(leaf_value, torch.float64, "leaf_value"), leaf_begin.numel(),
                                               float(learning_rate)))
        return score

    def boost_iteration(self, bins, label, score, bits_g, bits_h, seed, iteration, num_leaves, learning_rate,
                        min_data_in_leaf=20, min_sum_hessian=0.0, rounding=ROUND_STOCHASTIC, acc_width=0,
                        tree: Tree | None = None, group_size: int = 0, row_layout=ROWS_AUTO) -> Tree:
        """Loss derivatives, one tree and the score update on the device; `score` is updated in place.
        group_size > 0 selects the lambdarank loss (label = relevance), else binary cross-entropy."""
        self._sync_stream()
        tree = tree if tree is not None else self.new_tree()
        p = Params(bits_g, bits_h, rounding, num_leaves, min_data_in_leaf, acc_width, row_layout, seed, min_sum_hessian)
        tp = tree.ptrs()
        if group_size > 0:
            self._chk(self.lib.qgbdt_boost_iteration_lambdarank(
                self._h, self._bins(bins), _dev(label, torch.float32, "relevance"), int(group_size),
                _dev(score, torch.float32, "score"), C.byref(p), iteration, float(learning_rate), C.byref(tp),
                _dev(tree.row_idx, torch.int32, "row_idx")))
        else:
            self._chk(self.lib.qgbdt_boost_iteration(self._h, self._bins(bins),
                                                     _dev(label, torch.float32, "label"),
                                                     _dev(score, torch.float32, "score"), C.byref(p), iteration,
                                                     float(learning_rate), C.byref(tp),
                                                     _dev(tree.row_idx, torch.int32, "row_idx")))
        return tree

    # -- measurement -------------------------------------------------------------
    def set_profiling(self, on: bool):
        self._chk(self.lib.qgbdt_set_profiling(self._h, 1 if on else 0))

    def read_profile_roots(self):
        """(ms, launches) of the timed launches that were a tree's root build; call before read_profile."""
        ms = C.c_double(0); n = C.c_int64(0)
        self._chk(self.lib.qgbdt_read_profile_roots(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def read_profile(self):
        ms = C.c_double(0); n = C.c_int64(0); b = C.c_double(0)
        self._chk(self.lib.qgbdt_read_profile(self._h, C.byref(ms), C.byref(n), C.byref(b)))
        return ms.value, n.value, b.value


def _measure_stream_read(self, buf: torch.Tensor, reps: int = 10) -> float:
    """GB/s a plain 16-byte-load kernel reaches reading `buf` (device tensor) `reps` times."""
    self._sync_stream()
    if not buf.is_cuda or not buf.is_contiguous():
        raise ValueError("buf must be a contiguous device tensor")
    nbytes = buf.numel() * buf.element_size() // 16 * 16
    out = C.c_double(0)
    var = (C.c_int32 * 3)()
    self._chk(self.lib.qgbdt_measure_stream_read(self._h, C.c_void_p(buf.data_ptr()), C.c_int64(nbytes), int(reps),
                                                 C.byref(out), var))
    self.stream_read_variant = {"loads_in_flight": int(var[0]), "workgroups": int(var[1]), "non_temporal": bool(var[2])}
    return out.value


Context.measure_stream_read = _measure_stream_read


def _tree_stats(self):
    """(rounds, expanded nodes, committed splits, nodes) of the last grow_tree call."""
    out = (C.c_int32 * 4)()
    self._chk(self.lib.qgbdt_tree_stats(self._h, out))
    return tuple(int(x) for x in out)


Context.tree_stats = _tree_stats


def unpack_splits(raw: torch.Tensor):
    """Decodes qgbdt_split records (uint8 [n, 56]) into a list of dicts (host)."""
    import struct
    out = []
    for rec in raw.cpu().numpy():
        gain, feature, bin_, lg, lh, rg, rh, lc = struct.unpack("<diiqqqqq", rec.tobytes())
        out.append(dict(gain=gain, feature=feature, bin=bin_, GL=lg, HL=lh, GR=rg, HR=rh, cnt_left=lc))
    return out


def unpack_hist(hist: torch.Tensor, n_features: int, n_bins: int):
    """Packed int64 words [nb, F] -> (G int64 [F, nb], H int64 [F, nb]) on the host."""
    w = hist.cpu().view(n_bins, n_features).t().contiguous()
    return (w >> 32).numpy(), (w & 0xFFFFFFFF).numpy()
