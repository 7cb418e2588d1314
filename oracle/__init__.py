"""ctypes front end of the CPU oracle (``iwp_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the product package.
Argument marshalling only -- every step of the method runs in the C++ file.
All arrays are host numpy arrays, C-contiguous, float32 / uint32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "iwp_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

# IEEE binary32 with no contraction and no fast-math: the flags are part of the
# oracle's definition (Alg. 1 arithmetic read as plain fp32).
CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]


def build(force: bool = False) -> str:
    """Compile the oracle with g++; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", *CXXFLAGS, "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class Threshold(C.Structure):
    _fields_ = [("key", C.c_uint32), ("n_gt", C.c_uint32), ("n_eq_take", C.c_uint32)]


class Layer(C.Structure):
    _fields_ = [("offset", C.c_int64), ("n", C.c_uint32), ("k", C.c_uint32),
                ("out_offset", C.c_uint32), ("pad", C.c_uint32)]


_lib = None
_f32p = C.POINTER(C.c_float)
_u32p = C.POINTER(C.c_uint32)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.oracle_accumulate.argtypes = [_f32p, _f32p, C.c_uint64]
        L.oracle_accumulate.restype = None
        L.oracle_score.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float, _f32p]
        L.oracle_score.restype = None
        L.oracle_score_keys.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float, _u32p]
        L.oracle_score_keys.restype = None
        L.oracle_select.argtypes = [_f32p, C.c_uint32, C.c_uint32, _u32p, C.POINTER(Threshold)]
        L.oracle_select.restype = C.c_int
        L.oracle_take.argtypes = [_f32p, _u32p, C.c_uint32, _f32p]
        L.oracle_take.restype = None
        L.oracle_rank_of.argtypes = [_f32p, C.c_uint64, C.c_uint64]
        L.oracle_rank_of.restype = C.c_uint64
        L.oracle_compress_layer.argtypes = [_f32p, _f32p, _f32p, C.c_uint32, C.c_uint32, C.c_float,
                                            _u32p, _f32p, C.POINTER(Threshold)]
        L.oracle_compress_layer.restype = C.c_int
        L.oracle_select_threshold.argtypes = [_f32p, _f32p, C.c_uint32, C.c_uint32, C.c_float,
                                              C.POINTER(Threshold)]
        L.oracle_select_threshold.restype = C.c_int
        L.oracle_gather_sum.argtypes = [C.POINTER(_f32p), C.c_uint32, _u32p, C.c_uint64, _f32p]
        L.oracle_gather_sum.restype = None
        L.oracle_apply_sparse_update.argtypes = [_f32p, _u32p, _f32p, C.c_uint64, C.c_float,
                                                 C.POINTER(_f32p), C.c_uint32]
        L.oracle_apply_sparse_update.restype = None
        L.oracle_accumulate_momentum.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float]
        L.oracle_accumulate_momentum.restype = None
        L.oracle_step.argtypes = [_f32p, C.POINTER(_f32p), C.POINTER(_f32p), C.POINTER(C.c_uint8), C.c_float,
                                  C.c_uint32, C.POINTER(Layer), _u32p, C.c_uint32, C.c_float, C.c_float,
                                  _u32p, _f32p, _f32p, C.POINTER(Threshold)]
        L.oracle_step.restype = C.c_int
        _u8p = C.POINTER(C.c_uint8)
        L.oracle_mask_bytes.argtypes = [C.c_uint64]
        L.oracle_mask_bytes.restype = C.c_uint64
        L.oracle_mask_threshold.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float, C.c_float, _u8p]
        L.oracle_mask_threshold.restype = None
        L.oracle_mask_or.argtypes = [_u8p, _u8p, C.c_uint64]
        L.oracle_mask_or.restype = None
        L.oracle_mask_indices.argtypes = [_u8p, C.c_uint64, _u32p]
        L.oracle_mask_indices.restype = C.c_uint64
        L.oracle_step_threshold.argtypes = [_f32p, C.POINTER(_f32p), C.POINTER(_f32p), _u8p, C.c_float, C.c_uint32,
                                            C.POINTER(Layer), _u32p, C.c_uint32, _f32p, C.c_uint32, C.c_uint32,
                                            C.c_float, C.c_float, _u8p, _u32p, _u32p, _f32p, C.c_uint64,
                                            C.POINTER(C.c_uint64)]
        L.oracle_step_threshold.restype = C.c_int
        L.oracle_step_threshold_random.argtypes = [_f32p, C.POINTER(_f32p), C.POINTER(_f32p), _u8p, C.c_float, C.c_uint32,
                                                   C.POINTER(Layer), _u32p, C.c_uint32, _f32p, C.c_uint32,
                                                   C.c_uint64, C.c_uint64, C.c_uint32, C.c_float, C.c_float, _u8p,
                                                   _u32p, _u32p, _f32p, C.c_uint64, C.POINTER(C.c_uint64)]
        L.oracle_step_threshold_random.restype = C.c_int
        L.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
        L.oracle_uniform.restype = C.c_float
        L.oracle_mask_threshold_random.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float, C.c_float, C.c_uint64,
                                                   C.c_uint64, C.c_uint32, _u8p]
        L.oracle_mask_threshold_random.restype = None
        _f64p = C.POINTER(C.c_double)
        L.oracle_layer_stats.argtypes = [_f32p, _f32p, C.c_uint64, C.c_float, _f64p, _f64p]
        L.oracle_layer_stats.restype = None
        L.oracle_layerwise_threshold.argtypes = [C.c_double] * 5
        L.oracle_layerwise_threshold.restype = C.c_float
        L.oracle_step_layerwise.argtypes = [_f32p, C.POINTER(_f32p), C.POINTER(_f32p), _u8p, C.c_float, C.c_uint32,
                                            C.POINTER(Layer), _u32p, C.c_uint32, C.c_double, C.c_double, C.c_double,
                                            C.c_uint32, C.c_float, C.c_float, _f64p, _f32p, _u8p, _u32p, _u32p,
                                            _f32p, C.c_uint64, C.POINTER(C.c_uint64)]
        L.oracle_step_layerwise.restype = C.c_int
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous, "float32 C-contiguous array required"
    return a.ctypes.data_as(_f32p)


def _u32(a: np.ndarray):
    assert a.dtype == np.uint32 and a.flags.c_contiguous, "uint32 C-contiguous array required"
    return a.ctypes.data_as(_u32p)


def _ptr_array(arrays: Sequence[np.ndarray]):
    return (_f32p * len(arrays))(*[_f32(a) for a in arrays])


def accumulate(r: np.ndarray, g: np.ndarray) -> None:
    assert r.shape == g.shape
    lib().oracle_accumulate(_f32(r), _f32(g), r.size)


def accumulate_momentum(r: np.ndarray, g: np.ndarray, m: float) -> None:
    """M1: r <- (m * r) + g in place, two roundings."""
    lib().oracle_accumulate_momentum(_f32(r), _f32(g), r.size, C.c_float(m))


def score(w: np.ndarray, r: np.ndarray, eps: float) -> np.ndarray:
    s = np.empty(r.size, np.float32)
    lib().oracle_score(_f32(w), _f32(r), r.size, C.c_float(eps), _f32(s))
    return s


def score_keys(w: np.ndarray, r: np.ndarray, eps: float) -> np.ndarray:
    key = np.empty(r.size, np.uint32)
    lib().oracle_score_keys(_f32(w), _f32(r), r.size, C.c_float(eps), _u32(key))
    return key


def select(s: np.ndarray, k: int):
    """-> (idx ascending uint32[k], (key, n_gt, n_eq_take))."""
    idx = np.empty(k, np.uint32)
    thr = Threshold()
    rc = lib().oracle_select(_f32(s), s.size, k, _u32(idx), C.byref(thr))
    if rc:
        raise ValueError("oracle_select: rc=%d" % rc)
    return idx, (thr.key, thr.n_gt, thr.n_eq_take)


def take(r: np.ndarray, idx: np.ndarray) -> np.ndarray:
    val = np.empty(idx.size, np.float32)
    lib().oracle_take(_f32(r), _u32(idx), idx.size, _f32(val))
    return val


def rank_of(s: np.ndarray, i: int) -> int:
    return int(lib().oracle_rank_of(_f32(s), s.size, i))


def compress_layer(w: np.ndarray, g: np.ndarray, r: np.ndarray, k: int, eps: float):
    """r is updated in place.  -> (idx, val, (key, n_gt, n_eq_take))."""
    idx = np.empty(k, np.uint32)
    val = np.empty(k, np.float32)
    thr = Threshold()
    rc = lib().oracle_compress_layer(_f32(w), _f32(g), _f32(r), r.size, k, C.c_float(eps),
                                     _u32(idx), _f32(val), C.byref(thr))
    if rc:
        raise ValueError("oracle_compress_layer: rc=%d" % rc)
    return idx, val, (thr.key, thr.n_gt, thr.n_eq_take)


def select_threshold(w: np.ndarray, r: np.ndarray, k: int, eps: float):
    thr = Threshold()
    rc = lib().oracle_select_threshold(_f32(w), _f32(r), r.size, k, C.c_float(eps), C.byref(thr))
    if rc:
        raise ValueError("oracle_select_threshold: rc=%d" % rc)
    return (thr.key, thr.n_gt, thr.n_eq_take)


def gather_sum(residuals: Sequence[np.ndarray], idx: np.ndarray) -> np.ndarray:
    out = np.empty(idx.size, np.float32)
    lib().oracle_gather_sum(_ptr_array(residuals), len(residuals), _u32(idx), idx.size, _f32(out))
    return out


def apply_sparse_update(w: np.ndarray, idx: np.ndarray, s: np.ndarray, scale: float,
                        residuals: Sequence[np.ndarray]) -> None:
    lib().oracle_apply_sparse_update(_f32(w), _u32(idx), _f32(s), idx.size, C.c_float(scale),
                                     _ptr_array(residuals), len(residuals))


def layer_table(rows) -> "C.Array[Layer]":
    """rows: iterable of (offset, n, k, out_offset)."""
    rows = list(rows)
    tab = (Layer * len(rows))()
    for t, (off, n, k, oo) in zip(tab, rows):
        t.offset, t.n, t.k, t.out_offset, t.pad = int(off), int(n), int(k), int(oo), 0
    return tab


def step(w: np.ndarray, g: Sequence[np.ndarray], r: Sequence[np.ndarray], rows, leader: np.ndarray,
         eps: float, scale: float, accumulate_mask: Sequence[int] | None = None, momentum: float = 1.0):
    """One whole emulated step on flat host buffers; w and every r[p] are updated
    in place (momentum: M1 in place of O1).  -> (idx, val, sum, thr[n_layers] as uint32 array of shape (L, 3))."""
    rows = list(rows)
    tab = layer_table(rows)
    W = len(r)
    total = sum(int(k) for (_, _, k, _) in rows)
    idx = np.empty(total, np.uint32)
    val = np.empty(total, np.float32)
    sm = np.empty(total, np.float32)
    thr = (Threshold * len(rows))()
    acc = None
    if accumulate_mask is not None:
        acc = (C.c_uint8 * W)(*[1 if a else 0 for a in accumulate_mask])
    leader = np.ascontiguousarray(leader, np.uint32)
    rc = lib().oracle_step(_f32(w), _ptr_array(g), _ptr_array(r), acc, C.c_float(momentum), W, tab, _u32(leader), len(rows),
                           C.c_float(eps), C.c_float(scale), _u32(idx), _f32(val), _f32(sm), thr)
    if rc:
        raise ValueError("oracle_step: rc=%d" % rc)
    thr_np = np.array([(t.key, t.n_gt, t.n_eq_take) for t in thr], np.uint32).reshape(len(rows), 3)
    return idx, val, sm, thr_np


# ------------------------------------------------------------------ threshold mode

def _u8(a: np.ndarray):
    assert a.dtype == np.uint8 and a.flags.c_contiguous, "uint8 C-contiguous array required"
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def mask_bytes(n: int) -> int:
    return int(lib().oracle_mask_bytes(n))


def mask_threshold(w: np.ndarray, r: np.ndarray, eps: float, thr: float) -> np.ndarray:
    """Encoded mask (uint8, LSB first, padded to whole 32-bit words) of score > thr."""
    m = np.empty(mask_bytes(r.size), np.uint8)
    lib().oracle_mask_threshold(_f32(w), _f32(r), r.size, C.c_float(eps), C.c_float(thr), _u8(m))
    return m


def mask_or(acc: np.ndarray, m: np.ndarray) -> None:
    assert acc.size == m.size
    lib().oracle_mask_or(_u8(acc), _u8(m), acc.size)


def mask_indices(mask: np.ndarray, n: int) -> np.ndarray:
    idx = np.empty(n, np.uint32)
    c = int(lib().oracle_mask_indices(_u8(mask), n, _u32(idx)))
    return idx[:c].copy()


def step_threshold(w: np.ndarray, g: Sequence[np.ndarray], r: Sequence[np.ndarray], rows, leaders: np.ndarray,
                   thr: np.ndarray, eps: float, scale: float, max_pairs: int,
                   accumulate_mask: Sequence[int] | None = None, random: tuple | None = None, momentum: float = 1.0):
    """One whole threshold-mode step on flat host buffers; w and every r[p] are updated
    in place.  leaders: (n_layers, n_lead) uint32; thr: (n_layers,) float32, or
    (n_layers, n_lead) float32 (2-D) for one threshold per chosen node.
    random = (seed, step): with random gradient selection (Section 3.3).
    -> (mask bytes of all layers back to back, counts[n_layers], idx[total], sum[total])."""
    rows = list(rows)
    tab = layer_table(rows)
    W = len(r)
    leaders = np.ascontiguousarray(leaders, np.uint32).reshape(len(rows), -1)
    thr = np.ascontiguousarray(thr, np.float32)
    per_slot = 1 if thr.size == leaders.size and thr.ndim == 2 else 0
    assert per_slot or thr.size == len(rows)
    mask = np.zeros(sum(mask_bytes(int(n)) for (_, n, _, _) in rows), np.uint8)
    counts = np.zeros(len(rows), np.uint32)
    idx = np.empty(max_pairs, np.uint32)
    sm = np.empty(max_pairs, np.float32)
    total = C.c_uint64(0)
    acc = None
    if accumulate_mask is not None:
        acc = (C.c_uint8 * W)(*[1 if a else 0 for a in accumulate_mask])
    if random is None:
        rc = lib().oracle_step_threshold(_f32(w), _ptr_array(g), _ptr_array(r), acc, C.c_float(momentum), W, tab, _u32(leaders),
                                         leaders.shape[1], _f32(thr), per_slot, len(rows), C.c_float(eps),
                                         C.c_float(scale), _u8(mask), _u32(counts), _u32(idx), _f32(sm), max_pairs,
                                         C.byref(total))
    else:
        rc = lib().oracle_step_threshold_random(_f32(w), _ptr_array(g), _ptr_array(r), acc, C.c_float(momentum), W, tab, _u32(leaders),
                                                leaders.shape[1], _f32(thr), per_slot, int(random[0]), int(random[1]),
                                                len(rows), C.c_float(eps), C.c_float(scale), _u8(mask), _u32(counts),
                                                _u32(idx), _f32(sm), max_pairs, C.byref(total))
    if rc:
        raise ValueError("oracle_step_threshold: rc=%d" % rc)
    return mask, counts, idx[:total.value].copy(), sm[:total.value].copy()


def layer_stats(w: np.ndarray, r: np.ndarray, eps: float):
    """L1: (mean, population variance) of one node's importance over a layer, binary64."""
    m, v = C.c_double(0), C.c_double(0)
    lib().oracle_layer_stats(_f32(w), _f32(r), r.size, C.c_float(eps), C.byref(m), C.byref(v))
    return m.value, v.value


def layerwise_threshold(mean: float, var: float, alpha: float, beta: float, c: float) -> np.float32:
    """L2: the threshold Eq. 4 derives from a layer's statistics."""
    return np.float32(lib().oracle_layerwise_threshold(mean, var, alpha, beta, c))


def step_layerwise(w: np.ndarray, g: Sequence[np.ndarray], r: Sequence[np.ndarray], rows, leaders: np.ndarray,
                   alpha: float, beta: float, c: float, eps: float, scale: float, max_pairs: int,
                   accumulate_mask: Sequence[int] | None = None, momentum: float = 1.0):
    """One whole step with layer-wise thresholds.
    -> (stats[n_layers, n_lead, 2] float64, thr[n_layers, n_lead] float32, mask, counts, idx, sum)."""
    rows = list(rows)
    tab = layer_table(rows)
    W = len(r)
    leaders = np.ascontiguousarray(leaders, np.uint32).reshape(len(rows), -1)
    n_lead = leaders.shape[1]
    stats = np.zeros((len(rows), n_lead, 2), np.float64)
    thr = np.zeros((len(rows), n_lead), np.float32)
    mask = np.zeros(sum(mask_bytes(int(n)) for (_, n, _, _) in rows), np.uint8)
    counts = np.zeros(len(rows), np.uint32)
    idx = np.empty(max_pairs, np.uint32)
    sm = np.empty(max_pairs, np.float32)
    total = C.c_uint64(0)
    acc = None
    if accumulate_mask is not None:
        acc = (C.c_uint8 * W)(*[1 if a else 0 for a in accumulate_mask])
    rc = lib().oracle_step_layerwise(_f32(w), _ptr_array(g), _ptr_array(r), acc, C.c_float(momentum), W, tab, _u32(leaders), n_lead,
                                     alpha, beta, c, len(rows), C.c_float(eps), C.c_float(scale),
                                     stats.ctypes.data_as(C.POINTER(C.c_double)), _f32(thr), _u8(mask), _u32(counts),
                                     _u32(idx), _f32(sm), max_pairs, C.byref(total))
    if rc:
        raise ValueError("oracle_step_layerwise: rc=%d" % rc)
    return stats, thr, mask, counts, idx[:total.value].copy(), sm[:total.value].copy()


def philox4x32_10(ctr, key) -> np.ndarray:
    """S1: one Philox-4x32-10 block; ctr: 4 words, key: 2 words -> 4 words."""
    c = np.ascontiguousarray(ctr, np.uint32)
    k = np.ascontiguousarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().oracle_philox4x32_10(_u32(c), _u32(k), _u32(out))
    return out


def uniform(seed: int, step: int, layer: int, i: int) -> np.float32:
    """S1: the draw of element i of a layer at a step, a multiple of 2^-24 in [0, 1)."""
    return np.float32(lib().oracle_uniform(seed, step, layer, i))


def mask_threshold_random(w: np.ndarray, r: np.ndarray, eps: float, thr: float, seed: int, step: int,
                          layer: int) -> np.ndarray:
    """S2: encoded mask of one chosen node with random gradient selection."""
    mask = np.zeros(mask_bytes(r.size), np.uint8)
    lib().oracle_mask_threshold_random(_f32(w), _f32(r), r.size, C.c_float(eps), C.c_float(thr), seed, step, layer,
                                       _u8(mask))
    return mask
