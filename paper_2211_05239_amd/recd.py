"""Thin ctypes binding of librecd (the HIP library behind include/recd.h).

Argument marshalling only: every step of the path runs in the library's kernels.  torch is used
for device memory (tensors own the buffers) and for the stream handle.  There is no CPU fallback:
importing this module raises if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# RECD_LIB: load this build of the library instead (comparing two builds in one session)
LIB_PATH = os.environ.get("RECD_LIB") or os.path.join(_HERE, "librecd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2211_05239_amd.build` "
        "(hipcc, gfx950). There is no fallback path.")

_lib = C.CDLL(LIB_PATH)

RECD_OK = 0
RECD_EINVAL, RECD_ENOMEM, RECD_EHIP, RECD_EBOUNDS, RECD_ECAPACITY = -1, -2, -3, -4, -5
RECD_F32, RECD_F16, RECD_BF16 = 0, 1, 2
RECD_OPT_VALIDATE, RECD_OPT_WEAK_HASH, RECD_OPT_LONG_SEGMENT_CUT = 1, 2, 4
# not in the public header: launch-shape override of the gather-sum kernel (tuning runs, and the
# test that results do not depend on the launch shape)
_OPT_INTERNAL_TUNE_SEGSUM = 1003
# benchmark instrumentation (not in the public header): HIP-event brackets around single kernels
_OPT_INTERNAL_TIMING = 1004
# tests only (not in the public header): 0 = small batches take the general builder and the two-pass
# form of the one-pass forward too, 1 = default, 2 = the one-launch builder's waits are made to expire
_OPT_INTERNAL_SMALL_PATH = 1005
KERNEL_SLOTS = {"lookup_expand": 0, "expand_uncovered": 1, "lookup_unique": 2, "expand": 3, "kjt_lookup": 4,
                "hash_insert": 5, "grad_lists_sum": 6, "grad_rows_sum": 7, "emit": 8}
RECD_POOL_SUM, RECD_POOL_MEAN, RECD_POOL_MAX = 0, 1, 2
RECD_NOALLOC_MAX_LISTS = 65536
POOLING = {"sum": RECD_POOL_SUM, "mean": RECD_POOL_MEAN, "max": RECD_POOL_MAX}

EXPORTED = [
    "recd_create", "recd_destroy", "recd_set_option", "recd_last_error", "recd_status_string",
    "recd_workspace_bytes", "recd_build_ikjt", "recd_pooled_lookup_unique", "recd_expand_inverse",
    "recd_kjt_pooled_lookup", "recd_backward_dedup", "recd_sequence_lookup_unique",
    "recd_jagged_expand_inverse", "recd_kjt_sequence_lookup", "recd_build_ikjt_grouped",
    "recd_group_sum_unique", "recd_pooled_lookup_unique_mode", "recd_kjt_pooled_lookup_mode",
    "recd_build_partial_ikjt", "recd_pooled_lookup_partial", "recd_backward_sequence_dedup",
    "recd_backward_dedup_mode", "recd_build_ikjt_weighted", "recd_pooled_lookup_unique_weighted",
    "recd_kjt_pooled_lookup_weighted", "recd_backward_dedup_weighted", "recd_backward_dedup_max",
    "recd_last_ikjt_counts", "recd_backward_plan", "recd_backward_apply", "recd_build_ikjt_noalloc",
    "recd_build_ikjt_runs", "recd_ikjt_run_index", "recd_pooled_lookup_expand", "recd_last_ikjt_run_count",
    "recd_backward_plan_runs",
]

_vp = C.c_void_p
_lib.recd_create.argtypes = [C.POINTER(_vp), C.c_int, _vp, C.c_size_t]
_lib.recd_destroy.argtypes = [_vp]
_lib.recd_set_option.argtypes = [_vp, C.c_int, C.c_int64]
_lib.recd_last_error.argtypes = [_vp]
_lib.recd_last_error.restype = C.c_char_p
_lib.recd_status_string.argtypes = [C.c_int]
_lib.recd_status_string.restype = C.c_char_p
_lib.recd_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int, C.POINTER(C.c_size_t)]
_lib.recd_build_ikjt.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.recd_build_ikjt_noalloc.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.recd_build_ikjt_runs.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64] + [_vp] * 8
_lib.recd_ikjt_run_index.argtypes = [_vp, C.c_int, C.c_int64, _vp, _vp, _vp, _vp]
_lib.recd_pooled_lookup_expand.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, _vp,
                                           C.c_int64, _vp, _vp]
_lib.recd_pooled_lookup_unique.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, _vp,
                                           _vp, C.c_int64, _vp]
_lib.recd_expand_inverse.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, C.c_int, _vp, _vp, _vp, _vp]
_lib.recd_kjt_pooled_lookup.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp,
                                        _vp, _vp]
_lib.recd_backward_dedup.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp, _vp,
                                     C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float,
                                     _vp]
_lib.recd_backward_dedup_mode.argtypes = [_vp, C.c_int] + _lib.recd_backward_dedup.argtypes[1:]
_lib.recd_build_ikjt_weighted.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64] + [_vp] * 9
_lib.recd_pooled_lookup_unique_weighted.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, _vp,
                                                    _vp, _vp, C.c_int64, _vp]
_lib.recd_kjt_pooled_lookup_weighted.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int, _vp, _vp,
                                                 _vp, _vp, _vp, _vp]
_lib.recd_backward_dedup_weighted.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                              C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, _vp, C.c_float,
                                              C.c_float, _vp]
_lib.recd_backward_dedup_max.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp, _vp, C.c_int64,
                                         C.c_int64, _vp, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]
_lib.recd_last_ikjt_counts.argtypes = [_vp, _vp]
_lib.recd_backward_plan.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp, C.c_int64, C.c_int64,
                                    _vp, _vp]
_lib.recd_last_ikjt_run_count.argtypes = [_vp, _vp]
_lib.recd_backward_plan_runs.argtypes = [_vp, C.c_int, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp, C.c_int64, C.c_int64,
                                         _vp, C.c_int64, _vp, _vp]
_lib.recd_backward_apply.argtypes = [_vp, C.c_int, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]
_lib.recd_sequence_lookup_unique.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, _vp,
                                             _vp, C.c_int64, C.c_int64, _vp]
_lib.recd_jagged_expand_inverse.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, _vp,
                                            C.c_int64, _vp, _vp, _vp, _vp, _vp]
_lib.recd_kjt_sequence_lookup.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                          _vp, _vp, _vp, _vp, _vp]
_lib.recd_build_ikjt_grouped.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp,
                                         _vp, _vp, _vp, _vp, _vp]
_lib.recd_group_sum_unique.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, _vp,
                                       C.c_int64, _vp]
_lib.recd_pooled_lookup_unique_mode.argtypes = [_vp, C.c_int] + _lib.recd_pooled_lookup_unique.argtypes[1:]
_lib.recd_kjt_pooled_lookup_mode.argtypes = [_vp, C.c_int] + _lib.recd_kjt_pooled_lookup.argtypes[1:]
_lib.recd_build_partial_ikjt.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64] + [_vp] * 10
_lib.recd_pooled_lookup_partial.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp, C.c_int64,
                                            _vp, _vp, _vp, C.c_int64, _vp]
_lib.recd_backward_sequence_dedup.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, C.c_int, _vp, _vp, _vp, _vp, _vp,
                                              _vp, _vp, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, _vp, _vp,
                                              C.c_float, C.c_float, _vp]
_lib.recd_internal_kernel_ms.argtypes = [_vp, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                         C.POINTER(C.c_int)]
_lib.recd_internal_kernel_ms.restype = C.c_int
for _n in EXPORTED:
    if _n not in ("recd_last_error", "recd_status_string"):
        getattr(_lib, _n).restype = C.c_int

_DT = {torch.float32: RECD_F32, torch.float16: RECD_F16, torch.bfloat16: RECD_BF16}


class RecdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_lib.recd_status_string(status).decode()}: {message}")
        self.status = status


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def workspace_bytes(F: int, B: int, N: int, D: int) -> int:
    out = C.c_size_t(0)
    st = _lib.recd_workspace_bytes(F, B, N, D, C.byref(out))
    if st != RECD_OK:
        raise RecdError(st, "recd_workspace_bytes")
    return int(out.value)


class Context:
    """One recd_ctx bound to a device and to torch's current stream on it."""

    def __init__(self, device: int = 0, workspace_hint_bytes: int = 0, stream: Optional[int] = None):
        self._h = _vp()
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        st = _lib.recd_create(C.byref(self._h), device, _vp(stream), workspace_hint_bytes)
        if st != RECD_OK:
            raise RecdError(st, "recd_create failed")
        self.device = device
        self.options = {}

    def close(self):
        if self._h:
            _lib.recd_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != RECD_OK:
            raise RecdError(st, _lib.recd_last_error(self._h).decode())

    def kernel_ms(self, slot: str, reset: bool = True):
        """(average ms, median ms, count) of the event-bracketed launches of one kernel since the last
        reset (needs _OPT_INTERNAL_TIMING); synchronises the device."""
        avg, med, n = C.c_double(0), C.c_double(0), C.c_int(0)
        self._check(_lib.recd_internal_kernel_ms(self._h, KERNEL_SLOTS[slot], int(reset), C.byref(avg),
                                                 C.byref(med), C.byref(n)))
        return avg.value, med.value, n.value

    def set_option(self, opt: int, value: int):
        self._check(_lib.recd_set_option(self._h, opt, value))
        self.options[opt] = value   # what was last set (the library has no getter)

    # -- the five calls; tensors are caller-allocated device tensors ---------------------------
    def build_ikjt(self, F: int, B: int, values, offsets, u_values, u_offsets, inverse, feat_uoff,
                   want_counts: bool = False):
        host = (C.c_int64 * 2)(0, 0) if want_counts else None
        self._check(_lib.recd_build_ikjt(self._h, F, B, values.numel(), _ptr(values), _ptr(offsets),
                                         _ptr(u_values), _ptr(u_offsets), _ptr(inverse),
                                         _ptr(feat_uoff), host))
        return (int(host[0]), int(host[1])) if want_counts else None

    def build_ikjt_noalloc(self, F: int, B: int, values, offsets, u_values, u_offsets, inverse, feat_uoff):
        """build_ikjt on the library's static scratch array: allocates nothing, returns no counts."""
        self._check(_lib.recd_build_ikjt_noalloc(self._h, F, B, values.numel(), _ptr(values), _ptr(offsets),
                                                 _ptr(u_values), _ptr(u_offsets), _ptr(inverse),
                                                 _ptr(feat_uoff)))

    def build_ikjt_runs(self, F: int, B: int, values, offsets, u_values, u_offsets, inverse, feat_uoff,
                        run_index, want_counts: bool = False):
        """build_ikjt that also writes the batch's run index (int64 [3 * (F*B + 2)])."""
        assert run_index.numel() >= 3 * (F * B + 2)
        host = (C.c_int64 * 2)(0, 0) if want_counts else None
        self._check(_lib.recd_build_ikjt_runs(self._h, F, B, values.numel(), _ptr(values), _ptr(offsets),
                                              _ptr(u_values), _ptr(u_offsets), _ptr(inverse),
                                              _ptr(feat_uoff), _ptr(run_index), host))
        return (int(host[0]), int(host[1])) if want_counts else None

    def ikjt_run_index(self, F: int, B: int, inverse, feat_uoff, u_offsets, run_index):
        assert run_index.numel() >= 3 * (F * B + 2)
        self._check(_lib.recd_ikjt_run_index(self._h, F, B, _ptr(inverse), _ptr(feat_uoff), _ptr(u_offsets),
                                             _ptr(run_index)))

    def pooled_lookup_expand(self, tables, B: int, u_values, run_index, max_runs: int, pooled, out):
        F = len(tables)
        D = tables[0].shape[1] if F else pooled.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[pooled.dtype]
        assert out is None or out.dtype == pooled.dtype
        self._check(_lib.recd_pooled_lookup_expand(
            self._h, F, B, D, tdt, _DT[pooled.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(u_values), _ptr(run_index), max_runs, _ptr(pooled), _ptr(out)))

    def last_ikjt_counts(self):
        """(U, M) of the most recent build_ikjt / build_ikjt_weighted call; waits for that build only."""
        host = (C.c_int64 * 2)(0, 0)
        self._check(_lib.recd_last_ikjt_counts(self._h, host))
        return int(host[0]), int(host[1])

    @staticmethod
    def _table_array(tables: Sequence[torch.Tensor]):
        return (_vp * len(tables))(*[t.data_ptr() for t in tables])

    @staticmethod
    def _rows_array(tables: Sequence[torch.Tensor]):
        return (C.c_int64 * len(tables))(*[t.shape[0] for t in tables])

    def pooled_lookup_unique(self, tables, u_values, u_offsets, feat_uoff, max_lists: int, pooled,
                             mode: Optional[str] = None):
        F = len(tables)
        D = tables[0].shape[1] if F else pooled.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[pooled.dtype]
        if mode is not None:
            self._check(_lib.recd_pooled_lookup_unique_mode(
                self._h, POOLING[mode], F, D, tdt, _DT[pooled.dtype], self._table_array(tables),
                self._rows_array(tables), _ptr(u_values), _ptr(u_offsets), _ptr(feat_uoff), max_lists,
                _ptr(pooled)))
            return
        self._check(_lib.recd_pooled_lookup_unique(
            self._h, F, D, tdt, _DT[pooled.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(u_values), _ptr(u_offsets), _ptr(feat_uoff), max_lists, _ptr(pooled)))

    def expand_inverse(self, F: int, B: int, pooled, feat_uoff, inverse, out):
        D = pooled.shape[-1]
        assert out.dtype == pooled.dtype
        self._check(_lib.recd_expand_inverse(self._h, F, B, D, _DT[pooled.dtype], _ptr(pooled),
                                             _ptr(feat_uoff), _ptr(inverse), _ptr(out)))

    def kjt_pooled_lookup(self, tables, B: int, values, offsets, out, mode: Optional[str] = None):
        F = len(tables)
        D = tables[0].shape[1] if F else out.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[out.dtype]
        if mode is not None:
            self._check(_lib.recd_kjt_pooled_lookup_mode(
                self._h, POOLING[mode], F, B, D, tdt, _DT[out.dtype], self._table_array(tables),
                self._rows_array(tables), _ptr(values), _ptr(offsets), _ptr(out)))
            return
        self._check(_lib.recd_kjt_pooled_lookup(
            self._h, F, B, D, tdt, _DT[out.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(values), _ptr(offsets), _ptr(out)))

    def backward_dedup(self, F: int, B: int, grad_out, inverse, feat_uoff, u_values, u_offsets,
                       rows: Sequence[int], U_cap: int, M_cap: int, touched_rows, feat_roff, grad_rows,
                       tables=None, adagrad_state=None, lr: float = 0.0, eps: float = 0.0,
                       want_count: bool = False, mode: str = "sum"):
        D = grad_out.shape[-1]
        rows_arr = (C.c_int64 * len(rows))(*rows)
        tabs = self._table_array(tables) if tables is not None else None
        state = self._table_array(adagrad_state) if adagrad_state is not None else None
        host = (C.c_int64 * 1)(0) if want_count else None
        args = (F, B, D, _ptr(grad_out), _ptr(inverse), _ptr(feat_uoff), _ptr(u_values),
                _ptr(u_offsets), rows_arr, U_cap, M_cap, _ptr(touched_rows), _ptr(feat_roff), _ptr(grad_rows),
                tabs, state, lr, eps, host)
        if mode == "sum":
            self._check(_lib.recd_backward_dedup(self._h, *args))
        else:
            self._check(_lib.recd_backward_dedup_mode(self._h, POOLING[mode], *args))
        return int(host[0]) if want_count else None

    # -- per-id weights -----------------------------------------------------------------------
    def build_ikjt_weighted(self, F: int, B: int, values, weights, offsets, u_values, u_weights, u_offsets,
                            inverse, feat_uoff, want_counts: bool = False):
        host = (C.c_int64 * 2)(0, 0) if want_counts else None
        self._check(_lib.recd_build_ikjt_weighted(
            self._h, F, B, values.numel(), _ptr(values), _ptr(weights), _ptr(offsets), _ptr(u_values),
            _ptr(u_weights), _ptr(u_offsets), _ptr(inverse), _ptr(feat_uoff), host))
        return (int(host[0]), int(host[1])) if want_counts else None

    def pooled_lookup_unique_weighted(self, tables, u_values, u_weights, u_offsets, feat_uoff, max_lists: int,
                                      pooled):
        F = len(tables)
        D = tables[0].shape[1] if F else pooled.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[pooled.dtype]
        self._check(_lib.recd_pooled_lookup_unique_weighted(
            self._h, F, D, tdt, _DT[pooled.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(u_values), _ptr(u_weights), _ptr(u_offsets), _ptr(feat_uoff), max_lists, _ptr(pooled)))

    def kjt_pooled_lookup_weighted(self, tables, B: int, values, weights, offsets, out):
        F = len(tables)
        D = tables[0].shape[1] if F else out.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[out.dtype]
        self._check(_lib.recd_kjt_pooled_lookup_weighted(
            self._h, F, B, D, tdt, _DT[out.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(values), _ptr(weights), _ptr(offsets), _ptr(out)))

    def backward_dedup_weighted(self, F: int, B: int, grad_out, inverse, feat_uoff, u_values, u_weights,
                                u_offsets, rows: Sequence[int], U_cap: int, M_cap: int, touched_rows, feat_roff,
                                grad_rows, tables=None, adagrad_state=None, lr: float = 0.0, eps: float = 0.0,
                                want_count: bool = False):
        D = grad_out.shape[-1]
        rows_arr = (C.c_int64 * len(rows))(*rows)
        tabs = self._table_array(tables) if tables is not None else None
        state = self._table_array(adagrad_state) if adagrad_state is not None else None
        host = (C.c_int64 * 1)(0) if want_count else None
        self._check(_lib.recd_backward_dedup_weighted(
            self._h, F, B, D, _ptr(grad_out), _ptr(inverse), _ptr(feat_uoff), _ptr(u_values), _ptr(u_weights),
            _ptr(u_offsets), rows_arr, U_cap, M_cap, _ptr(touched_rows), _ptr(feat_roff), _ptr(grad_rows),
            tabs, state, lr, eps, host))
        return int(host[0]) if want_count else None

    def backward_plan(self, F: int, B: int, D: int, inverse, feat_uoff, u_values, u_offsets, rows: Sequence[int],
                      U_cap: int, M_cap: int, touched_rows, feat_roff):
        rows_arr = (C.c_int64 * len(rows))(*rows)
        self._check(_lib.recd_backward_plan(self._h, F, B, D, _ptr(inverse), _ptr(feat_uoff), _ptr(u_values),
                                            _ptr(u_offsets), rows_arr, U_cap, M_cap, _ptr(touched_rows),
                                            _ptr(feat_roff)))

    def last_ikjt_run_count(self) -> int:
        host = (C.c_int64 * 1)(0)
        self._check(_lib.recd_last_ikjt_run_count(self._h, host))
        return int(host[0])

    def backward_plan_runs(self, F: int, B: int, D: int, inverse, feat_uoff, u_values, u_offsets,
                           rows: Sequence[int], U_cap: int, M_cap: int, run_index, runs_cap: int, touched_rows,
                           feat_roff):
        rows_arr = (C.c_int64 * len(rows))(*rows)
        self._check(_lib.recd_backward_plan_runs(self._h, F, B, D, _ptr(inverse), _ptr(feat_uoff), _ptr(u_values),
                                                 _ptr(u_offsets), rows_arr, U_cap, M_cap, _ptr(run_index), runs_cap,
                                                 _ptr(touched_rows), _ptr(feat_roff)))

    def backward_apply(self, grad_out, grad_rows, tables=None, adagrad_state=None, lr: float = 0.0,
                       eps: float = 0.0, want_count: bool = False, mode: str = "sum"):
        tabs = self._table_array(tables) if tables is not None else None
        state = self._table_array(adagrad_state) if adagrad_state is not None else None
        host = (C.c_int64 * 1)(0) if want_count else None
        self._check(_lib.recd_backward_apply(self._h, POOLING[mode], _ptr(grad_out), _ptr(grad_rows), tabs, state,
                                             lr, eps, host))
        return int(host[0]) if want_count else None

    def backward_dedup_max(self, F: int, B: int, grad_out, inverse, feat_uoff, u_values, u_offsets,
                           rows: Sequence[int], U_cap: int, M_cap: int, lookup_tables, touched_rows, feat_roff,
                           grad_rows, tables=None, adagrad_state=None, lr: float = 0.0, eps: float = 0.0,
                           want_count: bool = False):
        D = grad_out.shape[-1]
        rows_arr = (C.c_int64 * len(rows))(*rows)
        tabs = self._table_array(tables) if tables is not None else None
        state = self._table_array(adagrad_state) if adagrad_state is not None else None
        host = (C.c_int64 * 1)(0) if want_count else None
        self._check(_lib.recd_backward_dedup_max(
            self._h, F, B, D, _ptr(grad_out), _ptr(inverse), _ptr(feat_uoff), _ptr(u_values), _ptr(u_offsets),
            rows_arr, U_cap, M_cap, self._table_array(lookup_tables), _ptr(touched_rows), _ptr(feat_roff),
            _ptr(grad_rows), tabs, state, lr, eps, host))
        return int(host[0]) if want_count else None

    # -- sequence (unpooled) features ---------------------------------------------------------
    def sequence_lookup_unique(self, tables, u_values, u_offsets, feat_uoff, max_lists: int, emb):
        F = len(tables)
        D = tables[0].shape[1] if F else emb.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[emb.dtype]
        self._check(_lib.recd_sequence_lookup_unique(
            self._h, F, D, tdt, _DT[emb.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(u_values), _ptr(u_offsets), _ptr(feat_uoff), max_lists, emb.shape[0], _ptr(emb)))

    def jagged_expand_inverse(self, F: int, B: int, emb, u_offsets, feat_uoff, inverse, offsets, out):
        D = emb.shape[-1]
        assert out.dtype == emb.dtype
        self._check(_lib.recd_jagged_expand_inverse(
            self._h, F, B, out.shape[0], D, _DT[emb.dtype], _ptr(emb), emb.shape[0], _ptr(u_offsets),
            _ptr(feat_uoff), _ptr(inverse), _ptr(offsets), _ptr(out)))

    def kjt_sequence_lookup(self, tables, B: int, values, offsets, out):
        F = len(tables)
        D = tables[0].shape[1] if F else out.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[out.dtype]
        self._check(_lib.recd_kjt_sequence_lookup(
            self._h, F, B, values.numel(), D, tdt, _DT[out.dtype], self._table_array(tables),
            self._rows_array(tables), _ptr(values), _ptr(offsets), _ptr(out)))

    # -- grouped IKJTs --------------------------------------------------------------------------
    def build_ikjt_grouped(self, F: int, B: int, group_off: Sequence[int], values, offsets, u_values,
                           u_offsets, inverse_g, group_uoff, feat_uoff, inverse_per_feature=None,
                           want_counts: bool = False):
        G = len(group_off) - 1
        goff = (C.c_int32 * (G + 1))(*group_off)
        host = (C.c_int64 * 3)(0, 0, 0) if want_counts else None
        self._check(_lib.recd_build_ikjt_grouped(
            self._h, F, B, values.numel(), G, goff, _ptr(values), _ptr(offsets), _ptr(u_values),
            _ptr(u_offsets), _ptr(inverse_g), _ptr(group_uoff), _ptr(feat_uoff),
            _ptr(inverse_per_feature), host))
        return (int(host[0]), int(host[1]), int(host[2])) if want_counts else None

    def group_sum_unique(self, F: int, group_off: Sequence[int], pooled, feat_uoff, group_uoff, combined):
        G = len(group_off) - 1
        goff = (C.c_int32 * (G + 1))(*group_off)
        assert combined.dtype == pooled.dtype
        self._check(_lib.recd_group_sum_unique(
            self._h, F, G, pooled.shape[-1], _DT[pooled.dtype], goff, _ptr(pooled), _ptr(feat_uoff),
            _ptr(group_uoff), combined.shape[0], _ptr(combined)))

    # -- partial IKJTs --------------------------------------------------------------------------
    def build_partial_ikjt(self, F: int, B: int, values, offsets, p_values, win_start, win_len, inverse,
                           feat_uoff, feat_poff, row_window=None, want_counts: bool = False):
        host = (C.c_int64 * 3)(0, 0, 0) if want_counts else None
        self._check(_lib.recd_build_partial_ikjt(
            self._h, F, B, values.numel(), _ptr(values), _ptr(offsets), _ptr(p_values), _ptr(win_start),
            _ptr(win_len), _ptr(inverse), _ptr(feat_uoff), _ptr(feat_poff), _ptr(row_window), host))
        return (int(host[0]), int(host[1]), int(host[2])) if want_counts else None

    def pooled_lookup_partial(self, tables, p_values, win_start, win_len, feat_uoff, max_lists: int, pooled):
        F = len(tables)
        D = tables[0].shape[1] if F else pooled.shape[-1]
        tdt = _DT[tables[0].dtype] if F else _DT[pooled.dtype]
        self._check(_lib.recd_pooled_lookup_partial(
            self._h, F, D, tdt, _DT[pooled.dtype], self._table_array(tables), self._rows_array(tables),
            _ptr(p_values), p_values.numel(), _ptr(win_start), _ptr(win_len), _ptr(feat_uoff), max_lists,
            _ptr(pooled)))

    def backward_sequence_dedup(self, F: int, B: int, grad_out, offsets, inverse, feat_uoff, u_values, u_offsets,
                                rows: Sequence[int], U_cap: int, M_cap: int, grad_emb, touched_rows, feat_roff,
                                grad_rows, tables=None, adagrad_state=None, lr: float = 0.0, eps: float = 0.0,
                                want_count: bool = False):
        D = grad_out.shape[-1]
        rows_arr = (C.c_int64 * len(rows))(*rows)
        tabs = self._table_array(tables) if tables is not None else None
        state = self._table_array(adagrad_state) if adagrad_state is not None else None
        host = (C.c_int64 * 1)(0) if want_count else None
        self._check(_lib.recd_backward_sequence_dedup(
            self._h, F, B, grad_out.shape[0], D, _ptr(grad_out), _ptr(offsets), _ptr(inverse), _ptr(feat_uoff),
            _ptr(u_values), _ptr(u_offsets), rows_arr, U_cap, M_cap, _ptr(grad_emb), _ptr(touched_rows),
            _ptr(feat_roff), _ptr(grad_rows), tabs, state, lr, eps, host))
        return int(host[0]) if want_count else None
