"""Thin Python binding of the C-ABI HIP library (``include/iwp.h``).

Argument marshalling only: torch tensors are used for device memory and
streams, every step of the method runs in the library's kernels.  The function
names are the library's.  A missing library is an error -- there is no CPU or
eager fallback behind these calls.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libiwp.so")

IWP_MAX_WORKERS = 32
IWP_OK, IWP_EINVAL, IWP_EALIGN, IWP_EWORKSPACE, IWP_ERANGE, IWP_EHIP, IWP_ESCRATCH = 0, -1, -2, -3, -4, -5, -6
IWP_STATIC_SCRATCH_BYTES = 64 << 20


class IwpError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(what)


class Layer(C.Structure):
    _fields_ = [("offset", C.c_int64), ("n", C.c_uint32), ("k", C.c_uint32),
                ("out_offset", C.c_uint32), ("pad", C.c_uint32)]


_lib = None
_vp = C.c_void_p


def load() -> C.CDLL:
    """Open libiwp.so (built beforehand by ``python -m paper_1901_01544_amd.build``
    or ``__graft_entry__.build()``).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_1901_01544_amd.build`; "
            "there is no fallback path" % LIB_PATH)
    # The device pointers and streams this binding passes come from torch, so the library has to
    # bind to the HIP runtime torch carries: torch is imported (its runtime loaded) before the library.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    L.iwp_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32]
    L.iwp_workspace_bytes.restype = C.c_size_t
    L.compress_layer.argtypes = [_vp, _vp, _vp, C.c_uint32, C.c_uint32, C.c_float, _vp, _vp, _vp, C.c_size_t, _vp]
    L.select_threshold.argtypes = [_vp, _vp, C.c_uint32, C.c_uint32, C.c_float, _vp, _vp, C.c_size_t, _vp]
    L.compact_pairs.argtypes = [_vp, _vp, C.c_uint32, C.c_float, _vp, C.c_uint32, _vp, _vp, _vp, C.c_size_t, _vp]
    L.gather_sum_at_indices.argtypes = [C.POINTER(_vp), C.c_uint32, _vp, C.c_uint32, _vp, _vp]
    L.apply_sparse_update.argtypes = [_vp, _vp, _vp, C.c_uint32, C.c_float, C.POINTER(_vp), C.c_uint32, _vp]
    L.iwp_plan_create.argtypes = [C.POINTER(Layer), C.c_uint32, C.POINTER(_vp)]
    L.iwp_plan_destroy.argtypes = [_vp]
    L.iwp_plan_destroy.restype = None
    L.iwp_plan_workspace_bytes.argtypes = [_vp]
    L.iwp_plan_workspace_bytes.restype = C.c_size_t
    L.iwp_plan_step_workspace_bytes.argtypes = [_vp, C.c_uint32]
    L.iwp_plan_step_workspace_bytes.restype = C.c_size_t
    L.iwp_step_segmented.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp, _vp, C.c_float,
                                     C.c_float, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.iwp_step_segmented.restype = C.c_int
    L.iwp_plan_set_momentum.argtypes = [_vp, C.c_float]
    L.iwp_plan_set_momentum.restype = C.c_int
    L.iwp_plan_mask_bytes.argtypes = [_vp]
    L.iwp_plan_mask_bytes.restype = C.c_size_t
    L.iwp_plan_threshold_workspace_bytes.argtypes = [_vp, C.c_uint32, C.c_uint32, C.c_uint32]
    L.iwp_plan_threshold_workspace_bytes.restype = C.c_size_t
    L.iwp_step_threshold_segmented.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp, C.c_uint32,
                                               _vp, C.c_float, C.c_float, _vp, _vp, _vp, _vp, C.c_uint32, _vp,
                                               C.c_size_t, _vp]
    L.iwp_step_threshold_segmented.restype = C.c_int
    L.iwp_step_threshold_random_segmented.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp,
                                                      C.c_uint32, _vp, C.c_uint64, C.c_uint64, C.c_float, C.c_float,
                                                      _vp, _vp, _vp, _vp, C.c_uint32, _vp, C.c_size_t, _vp]
    L.iwp_step_threshold_random_segmented.restype = C.c_int
    L.iwp_step_layerwise_segmented.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp, C.c_uint32,
                                               C.c_double, C.c_double, C.c_double, C.c_float, C.c_float, _vp, _vp,
                                               _vp, _vp, _vp, _vp, C.c_uint32, _vp, C.c_size_t, _vp]
    L.iwp_step_layerwise_segmented.restype = C.c_int
    L.iwp_plan_total_pairs.argtypes = [_vp]
    L.iwp_plan_total_pairs.restype = C.c_uint64
    L.compress_segmented.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp, _vp, C.c_float,
                                     _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.compress_segmented_static.argtypes = [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.c_uint32, _vp, _vp, C.c_float,
                                            _vp, _vp, _vp, _vp]
    L.compress_segmented_static.restype = C.c_int
    L.select_threshold_segmented.argtypes = [_vp, _vp, _vp, C.c_float, _vp, _vp, C.c_size_t, _vp]
    L.compact_pairs_segmented.argtypes = [_vp, _vp, _vp, C.c_float, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.iwp_score_keys.argtypes = [_vp, _vp, C.c_uint32, C.c_float, _vp, _vp]
    L.iwp_copy_f32.argtypes = [_vp, _vp, C.c_uint64, _vp]
    L.iwp_copy_f32.restype = C.c_int
    L.iwp_timing_enable.argtypes = [C.c_char_p, C.c_uint32]
    L.iwp_timing_enable.restype = C.c_int
    L.iwp_timing_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_uint32)]
    L.iwp_timing_collect.restype = C.c_int
    L.iwp_strerror.argtypes = [C.c_int]
    L.iwp_strerror.restype = C.c_char_p
    L.iwp_last_hip_error.argtypes = []
    L.iwp_last_hip_error.restype = C.c_char_p
    for name in ("compress_layer", "select_threshold", "compact_pairs", "gather_sum_at_indices",
                 "apply_sparse_update", "iwp_plan_create", "compress_segmented", "select_threshold_segmented",
                 "compact_pairs_segmented", "iwp_score_keys"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(rc: int, what: str) -> None:
    if rc != 0:
        L = load()
        msg = L.iwp_strerror(rc).decode()
        if rc == IWP_EHIP:
            msg += " (" + L.iwp_last_hip_error().decode() + ")"
        raise IwpError(rc, "%s: %s [%d]" % (what, msg, rc))


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "contiguous device tensor required"
    return t.data_ptr()


def _ptr_table(tensors: Sequence):
    return (_vp * max(1, len(tensors)))(*[_ptr(t) for t in tensors])


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


# ------------------------------------------------------------------ one layer

def workspace_bytes(n: int, k: int) -> int:
    return int(load().iwp_workspace_bytes(n, k))


def compress_layer(w, g, r, k: int, eps: float, idx_out, val_out, workspace, stream=None, n: Optional[int] = None):
    n = r.numel() if n is None else n
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().compress_layer(_ptr(w), _ptr(g), _ptr(r), n, k, eps, _ptr(idx_out), _ptr(val_out),
                                 _ptr(workspace), ws_bytes, _stream(stream)), "compress_layer")


def select_threshold(w, r, k: int, eps: float, thr_out, workspace, stream=None, n: Optional[int] = None):
    n = r.numel() if n is None else n
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().select_threshold(_ptr(w), _ptr(r), n, k, eps, _ptr(thr_out), _ptr(workspace), ws_bytes,
                                   _stream(stream)), "select_threshold")


def compact_pairs(w, r, eps: float, thr, k: int, idx_out, val_out, workspace, stream=None, n: Optional[int] = None):
    n = r.numel() if n is None else n
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().compact_pairs(_ptr(w), _ptr(r), n, eps, _ptr(thr), k, _ptr(idx_out), _ptr(val_out),
                                _ptr(workspace), ws_bytes, _stream(stream)), "compact_pairs")


# ------------------------------------------------------------------ exchange

def gather_sum_at_indices(residuals: Sequence, idx, k: int, sum_out, stream=None):
    _check(load().gather_sum_at_indices(_ptr_table(residuals), len(residuals), _ptr(idx), k, _ptr(sum_out),
                                        _stream(stream)), "gather_sum_at_indices")


def apply_sparse_update(w, idx, sum_, k: int, scale: float, residuals_to_clear: Sequence, stream=None):
    _check(load().apply_sparse_update(_ptr(w), _ptr(idx), _ptr(sum_), k, scale, _ptr_table(residuals_to_clear),
                                      len(residuals_to_clear), _stream(stream)), "apply_sparse_update")


# ------------------------------------------------------------------ all layers in one pass

class Plan:
    """Owner of an ``iwp_plan`` (layer table + its device image)."""

    def __init__(self, rows):
        rows = list(rows)
        tab = (Layer * max(1, len(rows)))()
        for t, (off, n, k, oo) in zip(tab, rows):
            t.offset, t.n, t.k, t.out_offset, t.pad = int(off), int(n), int(k), int(oo), 0
        handle = _vp()
        _check(load().iwp_plan_create(tab, len(rows), C.byref(handle)), "iwp_plan_create")
        self._h = handle
        self.n_layers = len(rows)
        self.workspace_bytes = int(load().iwp_plan_workspace_bytes(self._h))
        self.total_pairs = int(load().iwp_plan_total_pairs(self._h))

    def step_workspace_bytes(self, W: int) -> int:
        return int(load().iwp_plan_step_workspace_bytes(self._h, W))

    def set_momentum(self, m: float) -> None:
        _check(load().iwp_plan_set_momentum(self._h, m), "iwp_plan_set_momentum")

    @property
    def mask_bytes(self) -> int:
        return int(load().iwp_plan_mask_bytes(self._h))

    def threshold_workspace_bytes(self, W: int, n_lead: int, max_pairs: int) -> int:
        return int(load().iwp_plan_threshold_workspace_bytes(self._h, W, n_lead, max_pairs))

    def close(self):
        if getattr(self, "_h", None):
            load().iwp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def compress_segmented(plan: Plan, w, g: Sequence, r: Sequence, leader, eps: float, idx_out, val_out, thr_out,
                       workspace, stream=None, thr_hint=None):
    assert len(g) == len(r)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().compress_segmented(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r), _ptr(leader),
                                     _ptr(thr_hint), eps,
                                     _ptr(idx_out), _ptr(val_out), _ptr(thr_out), _ptr(workspace), ws_bytes,
                                     _stream(stream)), "compress_segmented")


def compress_segmented_static(plan: Plan, w, g: Sequence, r: Sequence, leader, eps: float, idx_out, val_out, thr_out,
                              stream=None, thr_hint=None):
    assert len(g) == len(r)
    _check(load().compress_segmented_static(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r), _ptr(leader),
                                            _ptr(thr_hint), eps, _ptr(idx_out), _ptr(val_out), _ptr(thr_out),
                                            _stream(stream)), "compress_segmented_static")


def step_segmented(plan: Plan, w, g: Sequence, r: Sequence, leader, eps: float, scale: float, idx_out, val_out,
                   sum_out, thr_out, workspace, stream=None, thr_hint=None):
    assert len(g) == len(r)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().iwp_step_segmented(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r), _ptr(leader),
                                     _ptr(thr_hint), eps, scale,
                                     _ptr(idx_out), _ptr(val_out), _ptr(sum_out), _ptr(thr_out), _ptr(workspace),
                                     ws_bytes, _stream(stream)), "iwp_step_segmented")


def step_threshold_segmented(plan: Plan, w, g: Sequence, r: Sequence, leaders, n_lead: int, thr, eps: float,
                             scale: float, mask_out, count_out, idx_out, sum_out, max_pairs: int, workspace,
                             stream=None):
    assert len(g) == len(r)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().iwp_step_threshold_segmented(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r), _ptr(leaders),
                                               n_lead, _ptr(thr), eps, scale, _ptr(mask_out), _ptr(count_out),
                                               _ptr(idx_out), _ptr(sum_out), max_pairs, _ptr(workspace), ws_bytes,
                                               _stream(stream)), "iwp_step_threshold_segmented")


def step_threshold_random_segmented(plan: Plan, w, g: Sequence, r: Sequence, leaders, n_lead: int, thr, seed: int,
                                    step: int, eps: float, scale: float, mask_out, count_out, idx_out, sum_out,
                                    max_pairs: int, workspace, stream=None):
    assert len(g) == len(r)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().iwp_step_threshold_random_segmented(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r),
                                                      _ptr(leaders), n_lead, _ptr(thr), seed, step, eps, scale,
                                                      _ptr(mask_out), _ptr(count_out), _ptr(idx_out), _ptr(sum_out),
                                                      max_pairs, _ptr(workspace), ws_bytes, _stream(stream)),
           "iwp_step_threshold_random_segmented")


def step_layerwise_segmented(plan: Plan, w, g: Sequence, r: Sequence, leaders, n_lead: int, alpha: float, beta: float,
                             c: float, eps: float, scale: float, stats_out, thr_out, mask_out, count_out, idx_out,
                             sum_out, max_pairs: int, workspace, stream=None):
    assert len(g) == len(r)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().iwp_step_layerwise_segmented(plan._h, _ptr(w), _ptr_table(g), _ptr_table(r), len(r), _ptr(leaders),
                                               n_lead, alpha, beta, c, eps, scale, _ptr(stats_out), _ptr(thr_out),
                                               _ptr(mask_out), _ptr(count_out), _ptr(idx_out), _ptr(sum_out),
                                               max_pairs, _ptr(workspace), ws_bytes, _stream(stream)),
           "iwp_step_layerwise_segmented")


def select_threshold_segmented(plan: Plan, w, r, eps: float, thr_out, workspace, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().select_threshold_segmented(plan._h, _ptr(w), _ptr(r), eps, _ptr(thr_out), _ptr(workspace),
                                             ws_bytes, _stream(stream)), "select_threshold_segmented")


def compact_pairs_segmented(plan: Plan, w, r, eps: float, thr, idx_out, val_out, workspace, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().compact_pairs_segmented(plan._h, _ptr(w), _ptr(r), eps, _ptr(thr), _ptr(idx_out), _ptr(val_out),
                                          _ptr(workspace), ws_bytes, _stream(stream)), "compact_pairs_segmented")


def score_keys(w, r, eps: float, key_out, stream=None):
    _check(load().iwp_score_keys(_ptr(w), _ptr(r), r.numel(), eps, _ptr(key_out), _stream(stream)), "iwp_score_keys")


def copy_f32(dst, src, stream=None):
    _check(load().iwp_copy_f32(_ptr(dst), _ptr(src), src.numel(), _stream(stream)), "iwp_copy_f32")


def timing_enable(kernel_name: str, max_launches: int = 0):
    _check(load().iwp_timing_enable(kernel_name.encode(), max_launches), "iwp_timing_enable")


def timing_collect():
    """-> (total milliseconds, launches) of the kernel named in timing_enable()."""
    ms, cnt = C.c_double(), C.c_uint32()
    _check(load().iwp_timing_collect(C.byref(ms), C.byref(cnt)), "iwp_timing_collect")
    return ms.value, cnt.value
