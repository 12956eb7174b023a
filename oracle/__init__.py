"""CPU oracle for the quantized-GBDT hot path: ctypes binding over qgbdt_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

All arrays are numpy, host memory.  Function names mirror the C entry points
(`qgbdt_ref_*`); each C function cites the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "qgbdt_oracle.c")
_LIB = os.path.join(_DIR, "libqgbdt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.qgbdt_ref_uniform24.restype = C.c_float
        _lib.qgbdt_ref_uniform24.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int]
        _lib.qgbdt_ref_max_rows_for_width.restype = C.c_int64
        _lib.qgbdt_ref_quantized_leaf_value.restype = C.c_double
        _lib.qgbdt_ref_quantized_leaf_value.argtypes = [C.c_int64, C.c_int64, C.c_float, C.c_float]
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key) -> np.ndarray:
    ctr = _c(ctr, np.uint32); key = _c(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().qgbdt_ref_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def uniform24(seed: int, iteration: int, row: int, stream: int) -> float:
    return float(lib().qgbdt_ref_uniform24(seed, iteration, row, stream))


def scales(g, h, bits_g: int, bits_h: int) -> np.ndarray:
    g = _c(g, np.float32); h = _c(h, np.float32)
    d = np.zeros(2, np.float32)
    _chk(lib().qgbdt_ref_scales(_p(g), _p(h), C.c_int64(g.size), bits_g, bits_h, _p(d)), "scales")
    return d


def quantize_gradients(g, h, bits_g: int, bits_h: int, seed: int, iteration: int, rounding: int = 0):
    """Returns (gq int8[N], hq uint8[N], delta float32[2])."""
    g = _c(g, np.float32); h = _c(h, np.float32)
    n = g.size
    gq = np.zeros(n, np.int8); hq = np.zeros(n, np.uint8); d = np.zeros(2, np.float32)
    _chk(lib().qgbdt_ref_quantize_gradients(_p(g), _p(h), C.c_int64(n), bits_g, bits_h,
                                            C.c_uint64(seed), C.c_uint32(iteration), rounding,
                                            _p(gq), _p(hq), _p(d)), "quantize_gradients")
    return gq, hq, d


def pack(G: int, H: int, w: int) -> int:
    word = C.c_int64(0)
    rc = lib().qgbdt_ref_pack(C.c_int64(G), C.c_int64(H), w, C.byref(word))
    if rc != 0:
        raise OverflowError(f"({G},{H}) does not fit {w}|{w} fields")
    return word.value


def unpack(word: int, w: int):
    G = C.c_int64(0); H = C.c_int64(0)
    lib().qgbdt_ref_unpack(C.c_int64(word), w, C.byref(G), C.byref(H))
    return G.value, H.value


def max_rows_for_width(bits_g: int, bits_h: int, w: int) -> int:
    return int(lib().qgbdt_ref_max_rows_for_width(bits_g, bits_h, w))


def _bins(bins):
    bins = np.ascontiguousarray(bins)
    if bins.dtype == np.uint8:
        return bins, 1
    if bins.dtype == np.uint16:
        return bins, 2
    raise TypeError("bins must be uint8 or uint16")


def build_histograms(bins, nb: int, gq, hq, row_idx=None, begin: int = 0, count: int | None = None):
    """Returns hist int64[F, nb, 2] (sum g~, sum h~)."""
    bins, bb = _bins(bins)
    N, F = bins.shape
    gq = _c(gq, np.int8); hq = _c(hq, np.uint8)
    if row_idx is not None:
        row_idx = _c(row_idx, np.int32)
        if count is None:
            count = row_idx.size - begin
    elif count is None:
        count = N - begin
    hist = np.zeros((F, nb, 2), np.int64)
    _chk(lib().qgbdt_ref_build_histograms(_p(bins), bb, F, nb, _p(gq), _p(hq),
                                          _p(row_idx) if row_idx is not None else None,
                                          C.c_int64(begin), C.c_int64(count), _p(hist)),
         "build_histograms")
    return hist


def subtract_histograms(parent, child):
    parent = _c(parent, np.int64); child = _c(child, np.int64)
    out = np.zeros_like(parent)
    _chk(lib().qgbdt_ref_subtract_histograms(_p(parent), _p(child), _p(out), C.c_int64(parent.size)),
         "subtract_histograms")
    return out


@dataclass
class Split:
    gain: float
    feature: int
    bin: int
    GL: int
    HL: int
    GR: int
    HR: int
    cnt_left: int


def find_best_split(hist, n_rows: int, Gs: int, Hs: int, delta_g, delta_h, min_data: int = 0,
                    min_sum_hess: float = 0.0) -> Split:
    hist = _c(hist, np.int64)
    F, nb, _ = hist.shape
    gain = C.c_double(0); f = C.c_int32(0); b = C.c_int32(0)
    st = np.zeros(5, np.int64)
    _chk(lib().qgbdt_ref_find_best_split(_p(hist), F, nb, C.c_int64(n_rows), C.c_int64(Gs),
                                         C.c_int64(Hs), C.c_float(delta_g), C.c_float(delta_h),
                                         C.c_int64(min_data), C.c_double(min_sum_hess),
                                         C.byref(gain), C.byref(f), C.byref(b), _p(st)),
         "find_best_split")
    return Split(gain.value, f.value, b.value, *[int(x) for x in st])


def partition_rows(bins, row_idx, begin: int, count: int, feature: int, bin: int):
    """Returns (new row_idx copy, n_left)."""
    bins, bb = _bins(bins)
    F = bins.shape[1]
    out = np.array(row_idx, dtype=np.int32, copy=True)
    if begin < 0 or count < 0 or begin + count > out.size:
        raise ValueError("slice outside row_idx")
    nl = C.c_int64(0)
    _chk(lib().qgbdt_ref_partition_rows(_p(bins), bb, F, _p(out), C.c_int64(begin),
                                        C.c_int64(count), feature, bin, C.byref(nl)),
         "partition_rows")
    return out, nl.value


def refit_leaves(g, h, row_idx, leaf_begin, leaf_count):
    g = _c(g, np.float32); h = _c(h, np.float32); row_idx = _c(row_idx, np.int32)
    leaf_begin = _c(leaf_begin, np.int64); leaf_count = _c(leaf_count, np.int64)
    out = np.zeros(leaf_begin.size, np.float64)
    _chk(lib().qgbdt_ref_refit_leaves(_p(g), _p(h), _p(row_idx), _p(leaf_begin), _p(leaf_count),
                                      int(leaf_begin.size), _p(out)), "refit_leaves")
    return out


def logistic_gradients(score, label):
    score = _c(score, np.float32); label = _c(label, np.float32)
    g = np.empty(score.size, np.float32); h = np.empty(score.size, np.float32)
    _chk(lib().qgbdt_ref_logistic_gradients(_p(score), _p(label), C.c_int64(score.size), _p(g), _p(h)), "logistic_gradients")
    return g, h


def lambdarank_gradients(score, label, group: int):
    score = _c(score, np.float32); label = _c(label, np.float32)
    g = np.empty(score.size, np.float32); h = np.empty(score.size, np.float32)
    _chk(lib().qgbdt_ref_lambdarank_gradients(_p(score), _p(label), C.c_int64(score.size), int(group), _p(g), _p(h)),
         "lambdarank_gradients")
    return g, h


def update_scores(score, row_idx, leaf_begin, leaf_count, leaf_value, lr: float):
    """Returns the updated copy of `score`."""
    out = np.array(score, dtype=np.float32, copy=True)
    row_idx = _c(row_idx, np.int32); leaf_begin = _c(leaf_begin, np.int64); leaf_count = _c(leaf_count, np.int64)
    leaf_value = _c(leaf_value, np.float64)
    _chk(lib().qgbdt_ref_update_scores(_p(out), _p(row_idx), _p(leaf_begin), _p(leaf_count), _p(leaf_value),
                                       int(leaf_begin.size), C.c_double(lr)), "update_scores")
    return out


def quantized_leaf_value(G: int, H: int, delta_g, delta_h) -> float:
    return float(lib().qgbdt_ref_quantized_leaf_value(G, H, C.c_float(delta_g), C.c_float(delta_h)))


@dataclass
class Tree:
    n_leaves: int
    split_leaf: np.ndarray
    split_feature: np.ndarray
    split_bin: np.ndarray
    split_gain: np.ndarray
    split_stats: np.ndarray      # [n_splits, 4] = GL, HL, GR, HR
    split_n_left: np.ndarray
    leaf_begin: np.ndarray
    leaf_count: np.ndarray
    leaf_G: np.ndarray
    leaf_H: np.ndarray
    leaf_value: np.ndarray
    leaf_value_quant: np.ndarray
    row_idx: np.ndarray
    delta: np.ndarray
    gq: np.ndarray
    hq: np.ndarray
    hist_units: int              # rows*features accumulated by histogram builds


def grow_tree(bins, nb: int, g, h, bits_g: int, bits_h: int, seed: int, iteration: int,
              num_leaves: int, min_data: int = 20, min_sum_hess: float = 0.0, rounding: int = 0,
              verify_sibling: bool = False) -> Tree:
    bins, bb = _bins(bins)
    N, F = bins.shape
    g = _c(g, np.float32); h = _c(h, np.float32)
    L = num_leaves
    n_leaves = C.c_int32(0)
    S = max(L - 1, 1)
    split_leaf = np.zeros(S, np.int32); split_feature = np.zeros(S, np.int32)
    split_bin = np.zeros(S, np.int32); split_gain = np.zeros(S, np.float64)
    split_stats = np.zeros((S, 4), np.int64); split_n_left = np.zeros(S, np.int64)
    leaf_begin = np.zeros(L, np.int64); leaf_count = np.zeros(L, np.int64)
    leaf_G = np.zeros(L, np.int64); leaf_H = np.zeros(L, np.int64)
    leaf_value = np.zeros(L, np.float64); leaf_value_quant = np.zeros(L, np.float64)
    row_idx = np.zeros(N, np.int32); delta = np.zeros(2, np.float32)
    gq = np.zeros(N, np.int8); hq = np.zeros(N, np.uint8)
    units = C.c_int64(0)
    _chk(lib().qgbdt_ref_grow_tree(
        _p(bins), bb, C.c_int64(N), F, nb, _p(g), _p(h), bits_g, bits_h, C.c_uint64(seed),
        C.c_uint32(iteration), rounding, L, C.c_int64(min_data), C.c_double(min_sum_hess),
        1 if verify_sibling else 0, C.byref(n_leaves), _p(split_leaf), _p(split_feature),
        _p(split_bin), _p(split_gain), _p(split_stats), _p(split_n_left), _p(leaf_begin),
        _p(leaf_count), _p(leaf_G), _p(leaf_H), _p(leaf_value), _p(leaf_value_quant),
        _p(row_idx), _p(delta), _p(gq), _p(hq), C.byref(units)), "grow_tree")
    nl = n_leaves.value
    ns = nl - 1
    return Tree(nl, split_leaf[:ns], split_feature[:ns], split_bin[:ns], split_gain[:ns],
                split_stats[:ns], split_n_left[:ns], leaf_begin[:nl], leaf_count[:nl],
                leaf_G[:nl], leaf_H[:nl], leaf_value[:nl], leaf_value_quant[:nl], row_idx, delta,
                gq, hq, units.value)
