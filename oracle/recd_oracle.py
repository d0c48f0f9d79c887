"""ctypes front-end of the plain C oracle (oracle/recd_oracle.c).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file; this module only marshals numpy arrays.  The two
closed-form functions of the paper's duplication model (Sec. 4.2 "Using IKJTs") are written
here because they are one line each.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

import numpy as np

from . import build as _build

# RECD_ORACLE_LIB: load this library instead (the mutation test of the pins points it at copies of
# the oracle with a planted mistake, in a process of its own).
_lib = C.CDLL(os.environ.get("RECD_ORACLE_LIB") or _build.build())

_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_f64p = C.POINTER(C.c_double)
_f32p = C.POINTER(C.c_float)

DTYPES = {"f32": 0, "f16": 1, "bf16": 2}

_lib.oracle_half_to_double.restype = C.c_double
_lib.oracle_half_to_double.argtypes = [C.c_uint16]
_lib.oracle_bf16_to_double.restype = C.c_double
_lib.oracle_bf16_to_double.argtypes = [C.c_uint16]


def _p(a: np.ndarray, t):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(t)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


class OracleError(ValueError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what}: precondition violated (code {rc})")


def half_to_double(bits: int) -> float:
    return float(_lib.oracle_half_to_double(C.c_uint16(bits)))


def bf16_to_double(bits: int) -> float:
    return float(_lib.oracle_bf16_to_double(C.c_uint16(bits)))


def check_kjt(F: int, B: int, values, offsets, rows=None) -> int:
    values, offsets = _i64(values), _i64(offsets)
    r = _i64(rows) if rows is not None else None
    return int(_lib.oracle_check_kjt(C.c_int(F), C.c_int64(B), C.c_int64(values.shape[0]),
                                     _p(values, _i64p), _p(offsets, _i64p),
                                     _p(r, _i64p) if r is not None else None))


def build_ikjt(F: int, B: int, values, offsets):
    """KJT -> IKJT (Sec. 4.2). Returns (u_values[M], u_offsets[U+1], inverse[F*B] int32, feat_uoff[F+1])."""
    values, offsets = _i64(values), _i64(offsets)
    _check(check_kjt(F, B, values, offsets), "build_ikjt")
    N, L = values.shape[0], F * B
    u_values = np.zeros(max(N, 1), dtype=np.int64)
    u_offsets = np.zeros(L + 1, dtype=np.int64)
    inverse = np.zeros(max(L, 1), dtype=np.int32)
    feat_uoff = np.zeros(F + 1, dtype=np.int64)
    rc = _lib.oracle_build_ikjt(C.c_int(F), C.c_int64(B), _p(values, _i64p), _p(offsets, _i64p),
                                _p(u_values, _i64p), _p(u_offsets, _i64p), _p(inverse, _i32p),
                                _p(feat_uoff, _i64p))
    _check(rc, "build_ikjt")
    U = int(feat_uoff[F])
    M = int(u_offsets[U])
    return u_values[:M].copy(), u_offsets[:U + 1].copy(), inverse[:L].copy(), feat_uoff


def build_ikjt_grouped(F: int, B: int, group_off, values, offsets):
    """KJT -> grouped IKJT (Sec. 4.2 "Grouped IKJTs"): group g = features [group_off[g], group_off[g+1])
    shares one inverse.  Returns (u_values[M], u_offsets[U+1], inverse_g[G*B] int32, group_uoff[G+1],
    feat_uoff[F+1]) with U = sum over features of their group's slot count."""
    values, offsets = _i64(values), _i64(offsets)
    group_off = np.ascontiguousarray(group_off, dtype=np.int32)
    G = group_off.shape[0] - 1
    _check(check_kjt(F, B, values, offsets), "build_ikjt_grouped")
    N, L = values.shape[0], F * B
    u_values = np.zeros(max(N, 1), dtype=np.int64)
    u_offsets = np.zeros(L + 1, dtype=np.int64)
    inverse_g = np.zeros(max(G * B, 1), dtype=np.int32)
    group_uoff = np.zeros(G + 1, dtype=np.int64)
    feat_uoff = np.zeros(F + 1, dtype=np.int64)
    rc = _lib.oracle_build_ikjt_grouped(C.c_int(F), C.c_int64(B), C.c_int(G), _p(group_off, _i32p),
                                        _p(values, _i64p), _p(offsets, _i64p), _p(u_values, _i64p),
                                        _p(u_offsets, _i64p), _p(inverse_g, _i32p), _p(group_uoff, _i64p),
                                        _p(feat_uoff, _i64p))
    _check(rc, "build_ikjt_grouped")
    U = int(feat_uoff[F])
    M = int(u_offsets[U])
    return u_values[:M].copy(), u_offsets[:U + 1].copy(), inverse_g[:G * B].copy(), group_uoff, feat_uoff


def build_partial_ikjt(F: int, B: int, values, offsets):
    """KJT -> partial IKJT (Sec. 7).  Returns (p_values[P], win_start[U], win_len[U], inverse[F*B] int32,
    feat_uoff[F+1], feat_poff[F+1]); see the C source for this build's reading of the construction."""
    values, offsets = _i64(values), _i64(offsets)
    _check(check_kjt(F, B, values, offsets), "build_partial_ikjt")
    N, L = values.shape[0], F * B
    p_values = np.zeros(max(N, 1), dtype=np.int64)
    win_start = np.zeros(max(L, 1), dtype=np.int64)
    win_len = np.zeros(max(L, 1), dtype=np.int64)
    inverse = np.zeros(max(L, 1), dtype=np.int32)
    feat_uoff = np.zeros(F + 1, dtype=np.int64)
    feat_poff = np.zeros(F + 1, dtype=np.int64)
    rc = _lib.oracle_build_partial_ikjt(C.c_int(F), C.c_int64(B), _p(values, _i64p), _p(offsets, _i64p),
                                        _p(p_values, _i64p), _p(win_start, _i64p), _p(win_len, _i64p),
                                        _p(inverse, _i32p), _p(feat_uoff, _i64p), _p(feat_poff, _i64p))
    _check(rc, "build_partial_ikjt")
    U, P = int(feat_uoff[F]), int(feat_poff[F])
    return (p_values[:P].copy(), win_start[:U].copy(), win_len[:U].copy(), inverse[:L].copy(), feat_uoff,
            feat_poff)


def partial_row_windows(F: int, B: int, win_start, win_len, inverse, feat_uoff) -> np.ndarray:
    """The paper's per-row inverse_lookup of a partial IKJT: int64 [F*B, 2] of [offset, length]."""
    u = np.repeat(_i64(feat_uoff)[:F], B) + np.asarray(inverse, dtype=np.int64)
    return np.stack([_i64(win_start)[u], _i64(win_len)[u]], axis=1) if F * B else np.zeros((0, 2), np.int64)


def _table_ptrs(tables: Sequence[np.ndarray], dtype: str):
    keep = []
    for t in tables:
        if dtype == "f32":
            assert t.dtype == np.float32
        elif dtype == "f16":
            assert t.dtype == np.float16
        else:
            assert t.dtype == np.uint16
        keep.append(np.ascontiguousarray(t))
    arr = (C.c_void_p * len(keep))(*[t.ctypes.data for t in keep])
    return arr, keep


def pooled_lookup(tables: Sequence[np.ndarray], dtype: str, values, offsets, list_off) -> np.ndarray:
    """Sum-pooled lookup (Sec. 2.2, Sec. 5) of the lists [list_off[f], list_off[f+1]) of each
    feature f in table f.  Returns float64 [L, D]."""
    F = len(tables)
    values, offsets, list_off = _i64(values), _i64(offsets), _i64(list_off)
    D = int(tables[0].shape[1]) if F else 1
    rows = _i64([t.shape[0] for t in tables])
    L = int(list_off[F]) if F else 0
    out = np.zeros((max(L, 1), D), dtype=np.float64)
    ptrs, keep = _table_ptrs(tables, dtype)
    rc = _lib.oracle_pooled_lookup(C.c_int(F), C.c_int(D), C.c_int(DTYPES[dtype]), ptrs,
                                   _p(rows, _i64p), _p(values, _i64p), _p(offsets, _i64p),
                                   _p(list_off, _i64p), _p(out, _f64p))
    _check(rc, "pooled_lookup")
    del keep
    return out[:L]


POOLING = {"sum": 0, "mean": 1, "max": 2}


def pooled_lookup_mode(mode: str, tables: Sequence[np.ndarray], dtype: str, values, offsets, list_off) -> np.ndarray:
    """Pooled lookup with the pooling function `mode` in {"sum", "mean", "max"} (Sec. 2.2); an empty
    list pools to zero.  Same arguments and result layout as pooled_lookup."""
    F = len(tables)
    values, offsets, list_off = _i64(values), _i64(offsets), _i64(list_off)
    D = int(tables[0].shape[1]) if F else 1
    rows = _i64([t.shape[0] for t in tables])
    L = int(list_off[F]) if F else 0
    out = np.zeros((max(L, 1), D), dtype=np.float64)
    ptrs, keep = _table_ptrs(tables, dtype)
    rc = _lib.oracle_pooled_lookup_mode(C.c_int(POOLING[mode]), C.c_int(F), C.c_int(D), C.c_int(DTYPES[dtype]),
                                        ptrs, _p(rows, _i64p), _p(values, _i64p), _p(offsets, _i64p),
                                        _p(list_off, _i64p), _p(out, _f64p))
    _check(rc, "pooled_lookup_mode")
    del keep
    return out[:L]


def kjt_pooled_lookup(tables, dtype: str, B: int, values, offsets) -> np.ndarray:
    """Non-deduplicated lookup over every row of the batch. float64 [F, B, D]."""
    F = len(tables)
    list_off = np.arange(F + 1, dtype=np.int64) * B
    out = pooled_lookup(tables, dtype, values, offsets, list_off)
    return out.reshape(F, B, -1)


def expand_inverse(F: int, B: int, pooled: np.ndarray, feat_uoff, inverse) -> np.ndarray:
    """out[f,b,:] = pooled[feat_uoff[f] + inverse[f,b], :]  (Sec. 5 index_select). float64 [F,B,D]."""
    pooled = np.ascontiguousarray(pooled, dtype=np.float64)
    D = pooled.shape[1]
    feat_uoff = _i64(feat_uoff)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    out = np.zeros((F, B, D), dtype=np.float64)
    rc = _lib.oracle_expand_inverse(C.c_int(F), C.c_int64(B), C.c_int(D), _p(pooled, _f64p),
                                    _p(feat_uoff, _i64p), _p(inverse, _i32p), _p(out, _f64p))
    _check(rc, "expand_inverse")
    return out


def first_rows(F: int, B: int, inverse, feat_uoff) -> np.ndarray:
    """first_row[u] = f*B + b of the first row of feature f that names unique list u (-1: none)."""
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    feat_uoff = _i64(feat_uoff)
    out = np.full(max(int(feat_uoff[F]), 1), -1, dtype=np.int64)
    inv = inverse if inverse.size else np.zeros(1, dtype=np.int32)
    _check(_lib.oracle_first_rows(C.c_int(F), C.c_int64(B), _p(inv, _i32p), _p(feat_uoff, _i64p),
                                  _p(out, _i64p)), "first_rows")
    return out[:int(feat_uoff[F])]


def run_index(F: int, B: int, inverse, feat_uoff, u_offsets):
    """Runs of adjacent rows naming one unique list, in (feature, row) order.  Returns
    (run_row[R+1], run_list[R], run_first[R], run_start[R], run_ids[R]); run_row[R] = F*B."""
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    feat_uoff, u_offsets = _i64(feat_uoff), _i64(u_offsets)
    L = F * B
    row = np.zeros(L + 1, dtype=np.int64)
    lst = np.zeros(max(L, 1), dtype=np.int64)
    first = np.zeros(max(L, 1), dtype=np.int32)
    start = np.zeros(max(L, 1), dtype=np.int64)
    ids = np.zeros(max(L, 1), dtype=np.int64)
    inv = inverse if inverse.size else np.zeros(1, dtype=np.int32)
    _lib.oracle_run_index.restype = C.c_int64
    R = int(_lib.oracle_run_index(C.c_int(F), C.c_int64(B), _p(inv, _i32p), _p(feat_uoff, _i64p),
                                  _p(u_offsets, _i64p), _p(row, _i64p), _p(lst, _i64p), _p(first, _i32p),
                                  _p(start, _i64p), _p(ids, _i64p)))
    if R < 0:
        raise OracleError(f"run_index: precondition violated (code {R})")
    return row[:R + 1], lst[:R], first[:R], start[:R], ids[:R]


def pack_run_index(row, lst, first, start, ids, U: int, M: int) -> np.ndarray:
    """The run index in the library's int64 triples: {R, U, M}, then per run
    {row | (list | first << 31) << 32, ids at, ids}, then the closing entry {F*B, M, 0}."""
    R = len(lst)
    out = np.zeros(3 * (R + 2), dtype=np.uint64)
    out[0:3] = (R, U, M)
    uf = lst.astype(np.uint64) | (first.astype(np.uint64) << np.uint64(31))
    out[3:3 + 3 * R:3] = row[:R].astype(np.uint64) | (uf << np.uint64(32))
    out[4:4 + 3 * R:3] = start.astype(np.uint64)
    out[5:5 + 3 * R:3] = ids.astype(np.uint64)
    out[3 + 3 * R:6 + 3 * R] = (int(row[R]), M, 0)
    return out.view(np.int64)


def group_sum(group_off, pooled: np.ndarray, feat_uoff, group_uoff) -> np.ndarray:
    """Element-wise sum over the features of every group on the unique rows (Sec. 5 "Deduplicated
    Pooling").  pooled float64 [U, D] -> float64 [sum of U_g, D]."""
    group_off = np.ascontiguousarray(group_off, dtype=np.int32)
    feat_uoff, group_uoff = _i64(feat_uoff), _i64(group_uoff)
    pooled = np.ascontiguousarray(pooled, dtype=np.float64)
    G, F, D = group_off.shape[0] - 1, feat_uoff.shape[0] - 1, pooled.shape[1]
    out = np.zeros((max(int(group_uoff[G]), 1), D), dtype=np.float64)
    rc = _lib.oracle_group_sum(C.c_int(F), C.c_int(G), C.c_int(D), _p(group_off, _i32p), _p(pooled, _f64p),
                               _p(feat_uoff, _i64p), _p(group_uoff, _i64p), _p(out, _f64p))
    _check(rc, "group_sum")
    return out[:int(group_uoff[G])]


def sequence_lookup(tables: Sequence[np.ndarray], dtype: str, values, offsets, list_off) -> np.ndarray:
    """Per-id activations (Sec. 2.2, Sec. 5): emb[j,:] = W_f[values[j],:] for every position j of the
    lists [list_off[f], list_off[f+1]) of feature f.  Returns float64 [len(values), D]."""
    F = len(tables)
    values, offsets, list_off = _i64(values), _i64(offsets), _i64(list_off)
    D = int(tables[0].shape[1]) if F else 1
    rows = _i64([t.shape[0] for t in tables])
    emb = np.zeros((max(values.shape[0], 1), D), dtype=np.float64)
    ptrs, keep = _table_ptrs(tables, dtype)
    rc = _lib.oracle_sequence_lookup(C.c_int(F), C.c_int(D), C.c_int(DTYPES[dtype]), ptrs,
                                     _p(rows, _i64p), _p(values, _i64p), _p(offsets, _i64p),
                                     _p(list_off, _i64p), _p(emb, _f64p))
    _check(rc, "sequence_lookup")
    del keep
    return emb[:values.shape[0]]


def jagged_expand(F: int, B: int, emb: np.ndarray, u_offsets, feat_uoff, inverse, offsets) -> np.ndarray:
    """Jagged index select (Sec. 5): out[offsets[f*B+b] + t, :] = emb[u_offsets[u] + t, :] with
    u = feat_uoff[f] + inverse[f,b].  Returns float64 [N, D] in the KJT's own jagged layout."""
    emb = np.ascontiguousarray(emb, dtype=np.float64)
    D = emb.shape[1]
    u_offsets, feat_uoff, offsets = _i64(u_offsets), _i64(feat_uoff), _i64(offsets)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    N = int(offsets[F * B])
    out = np.zeros((max(N, 1), D), dtype=np.float64)
    rc = _lib.oracle_jagged_expand(C.c_int(F), C.c_int64(B), C.c_int(D), _p(emb, _f64p),
                                   _p(u_offsets, _i64p), _p(feat_uoff, _i64p), _p(inverse, _i32p),
                                   _p(offsets, _i64p), _p(out, _f64p))
    _check(rc, "jagged_expand")
    return out[:N]


def backward_dedup(F: int, B: int, grad_out: np.ndarray, inverse, feat_uoff, u_values, u_offsets,
                   mode: str = "sum"):
    """Returns (touched_rows[R] int64, feat_roff[F+1], grad_rows[R,D] float64); mode "sum" or "mean"."""
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
    D = grad_out.shape[-1]
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    feat_uoff, u_values, u_offsets = _i64(feat_uoff), _i64(u_values), _i64(u_offsets)
    M = u_values.shape[0]
    touched = np.zeros(max(M, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(M, 1), D), dtype=np.float64)
    fn = {"sum": _lib.oracle_backward_dedup, "mean": _lib.oracle_backward_dedup_mean}[mode]
    rc = fn(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p), _p(inverse, _i32p), _p(feat_uoff, _i64p),
            _p(u_values, _i64p), _p(u_offsets, _i64p), _p(touched, _i64p), _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_dedup")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def backward_kjt(F: int, B: int, grad_out: np.ndarray, values, offsets, mode: str = "sum"):
    """Same gradient computed from the KJT alone. Returns (touched_rows, feat_roff, grad_rows)."""
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
    D = grad_out.shape[-1]
    values, offsets = _i64(values), _i64(offsets)
    N = values.shape[0]
    touched = np.zeros(max(N, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(N, 1), D), dtype=np.float64)
    fn = {"sum": _lib.oracle_backward_kjt, "mean": _lib.oracle_backward_kjt_mean}[mode]
    rc = fn(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p), _p(values, _i64p), _p(offsets, _i64p),
            _p(touched, _i64p), _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_kjt")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def backward_sequence_dedup(F: int, B: int, grad_out: np.ndarray, offsets, inverse, feat_uoff, u_values,
                            u_offsets):
    """Backward of jagged expand + unpooled lookup; grad_out fp32 [N, D], one row per KJT position.
    Returns (touched_rows, feat_roff, grad_rows float64 [R, D])."""
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
    D = grad_out.shape[-1]
    offsets, feat_uoff, u_values, u_offsets = _i64(offsets), _i64(feat_uoff), _i64(u_values), _i64(u_offsets)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    M = u_values.shape[0]
    touched = np.zeros(max(M, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(M, 1), D), dtype=np.float64)
    rc = _lib.oracle_backward_sequence_dedup(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p),
                                             _p(offsets, _i64p), _p(inverse, _i32p), _p(feat_uoff, _i64p),
                                             _p(u_values, _i64p), _p(u_offsets, _i64p), _p(touched, _i64p),
                                             _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_sequence_dedup")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def backward_sequence_kjt(F: int, B: int, grad_out: np.ndarray, values, offsets):
    """The same gradient computed from the KJT alone (gradient of a plain embedding lookup)."""
    grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
    D = grad_out.shape[-1]
    values, offsets = _i64(values), _i64(offsets)
    N = values.shape[0]
    touched = np.zeros(max(N, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(N, 1), D), dtype=np.float64)
    rc = _lib.oracle_backward_sequence_kjt(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p),
                                           _p(values, _i64p), _p(offsets, _i64p), _p(touched, _i64p),
                                           _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_sequence_kjt")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


# ---- per-id weights (this build's reading: a weighted KJT holds one fp32 weight beside every id) ----
def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def build_ikjt_weighted(F: int, B: int, values, weights, offsets):
    """Weighted KJT -> IKJT: rows are duplicates iff ids and weight bit patterns agree position by
    position.  Returns (u_values[M], u_weights[M] float32, u_offsets[U+1], inverse[F*B], feat_uoff[F+1])."""
    values, offsets, weights = _i64(values), _i64(offsets), _f32(weights)
    _check(check_kjt(F, B, values, offsets), "build_ikjt_weighted")
    assert weights.shape == values.shape
    N, L = values.shape[0], F * B
    u_values = np.zeros(max(N, 1), dtype=np.int64)
    u_weights = np.zeros(max(N, 1), dtype=np.float32)
    u_offsets = np.zeros(L + 1, dtype=np.int64)
    inverse = np.zeros(max(L, 1), dtype=np.int32)
    feat_uoff = np.zeros(F + 1, dtype=np.int64)
    rc = _lib.oracle_build_ikjt_weighted(C.c_int(F), C.c_int64(B), _p(values, _i64p), _p(weights, _f32p),
                                         _p(offsets, _i64p), _p(u_values, _i64p), _p(u_weights, _f32p),
                                         _p(u_offsets, _i64p), _p(inverse, _i32p), _p(feat_uoff, _i64p))
    _check(rc, "build_ikjt_weighted")
    U = int(feat_uoff[F])
    M = int(u_offsets[U])
    return u_values[:M].copy(), u_weights[:M].copy(), u_offsets[:U + 1].copy(), inverse[:L].copy(), feat_uoff


def pooled_lookup_weighted(tables: Sequence[np.ndarray], dtype: str, values, weights, offsets, list_off) -> np.ndarray:
    """out[l] = sum_j weights[j] * W_f[values[j]] over the ids of list l.  Returns float64 [L, D]."""
    F = len(tables)
    values, offsets, list_off, weights = _i64(values), _i64(offsets), _i64(list_off), _f32(weights)
    D = int(tables[0].shape[1]) if F else 1
    rows = _i64([t.shape[0] for t in tables])
    L = int(list_off[F]) if F else 0
    out = np.zeros((max(L, 1), D), dtype=np.float64)
    ptrs, keep = _table_ptrs(tables, dtype)
    rc = _lib.oracle_pooled_lookup_weighted(C.c_int(F), C.c_int(D), C.c_int(DTYPES[dtype]), ptrs, _p(rows, _i64p),
                                            _p(values, _i64p), _p(weights, _f32p), _p(offsets, _i64p),
                                            _p(list_off, _i64p), _p(out, _f64p))
    _check(rc, "pooled_lookup_weighted")
    del keep
    return out[:L]


def backward_dedup_weighted(F: int, B: int, grad_out: np.ndarray, inverse, feat_uoff, u_values, u_weights,
                            u_offsets):
    """Backward of expand + weighted pooled lookup.  Returns (touched_rows, feat_roff, grad_rows float64)."""
    grad_out = _f32(grad_out)
    D = grad_out.shape[-1]
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    feat_uoff, u_values, u_offsets, u_weights = _i64(feat_uoff), _i64(u_values), _i64(u_offsets), _f32(u_weights)
    M = u_values.shape[0]
    touched = np.zeros(max(M, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(M, 1), D), dtype=np.float64)
    rc = _lib.oracle_backward_dedup_weighted(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p),
                                             _p(inverse, _i32p), _p(feat_uoff, _i64p), _p(u_values, _i64p),
                                             _p(u_weights, _f32p), _p(u_offsets, _i64p), _p(touched, _i64p),
                                             _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_dedup_weighted")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def backward_kjt_weighted(F: int, B: int, grad_out: np.ndarray, values, weights, offsets):
    """The same gradient from the weighted KJT alone."""
    grad_out = _f32(grad_out)
    D = grad_out.shape[-1]
    values, offsets, weights = _i64(values), _i64(offsets), _f32(weights)
    N = values.shape[0]
    touched = np.zeros(max(N, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(N, 1), D), dtype=np.float64)
    rc = _lib.oracle_backward_kjt_weighted(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p),
                                           _p(values, _i64p), _p(weights, _f32p), _p(offsets, _i64p),
                                           _p(touched, _i64p), _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_kjt_weighted")
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def _f32_table_ptrs(tables):
    keep = [np.ascontiguousarray(t, dtype=np.float32) for t in tables]
    return (C.c_void_p * len(keep))(*[t.ctypes.data for t in keep]), keep


def backward_dedup_max(F: int, B: int, grad_out: np.ndarray, inverse, feat_uoff, u_values, u_offsets, tables):
    """Backward of expand + max-pooled lookup (fp32 tables of the forward pass; the first position
    wins a tie).  Returns (touched_rows, feat_roff, grad_rows float64)."""
    grad_out = _f32(grad_out)
    D = grad_out.shape[-1]
    inverse = np.ascontiguousarray(inverse, dtype=np.int32)
    feat_uoff, u_values, u_offsets = _i64(feat_uoff), _i64(u_values), _i64(u_offsets)
    M = u_values.shape[0]
    touched = np.zeros(max(M, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(M, 1), D), dtype=np.float64)
    ptrs, keep = _f32_table_ptrs(tables)
    rc = _lib.oracle_backward_dedup_max(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p), _p(inverse, _i32p),
                                        _p(feat_uoff, _i64p), _p(u_values, _i64p), _p(u_offsets, _i64p), ptrs,
                                        _p(touched, _i64p), _p(feat_roff, _i64p), _p(grad_rows, _f64p))
    _check(rc, "backward_dedup_max")
    del keep
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def backward_kjt_max(F: int, B: int, grad_out: np.ndarray, values, offsets, tables):
    """The same gradient from the KJT alone."""
    grad_out = _f32(grad_out)
    D = grad_out.shape[-1]
    values, offsets = _i64(values), _i64(offsets)
    N = values.shape[0]
    touched = np.zeros(max(N, 1), dtype=np.int64)
    feat_roff = np.zeros(F + 1, dtype=np.int64)
    grad_rows = np.zeros((max(N, 1), D), dtype=np.float64)
    ptrs, keep = _f32_table_ptrs(tables)
    rc = _lib.oracle_backward_kjt_max(C.c_int(F), C.c_int64(B), C.c_int(D), _p(grad_out, _f32p), _p(values, _i64p),
                                      _p(offsets, _i64p), ptrs, _p(touched, _i64p), _p(feat_roff, _i64p),
                                      _p(grad_rows, _f64p))
    _check(rc, "backward_kjt_max")
    del keep
    R = int(feat_roff[F])
    return touched[:R].copy(), feat_roff, grad_rows[:R].copy()


def rowwise_adagrad(grad_rows, w_rows, m_rows, lr: float, eps: float) -> Tuple[np.ndarray, np.ndarray]:
    """Row-wise Adagrad on the touched rows: returns (w_new[R,D], m_new[R]) in float64."""
    grad_rows = np.ascontiguousarray(grad_rows, dtype=np.float64)
    w_rows = np.ascontiguousarray(w_rows, dtype=np.float64)
    m_rows = np.ascontiguousarray(m_rows, dtype=np.float64)
    R, D = grad_rows.shape
    w_new = np.zeros((max(R, 1), D), dtype=np.float64)
    m_new = np.zeros(max(R, 1), dtype=np.float64)
    rc = _lib.oracle_rowwise_adagrad(C.c_int64(R), C.c_int(D), _p(grad_rows, _f64p),
                                     _p(w_rows, _f64p), _p(m_rows, _f64p), C.c_double(lr),
                                     C.c_double(eps), _p(w_new, _f64p), _p(m_new, _f64p))
    _check(rc, "rowwise_adagrad")
    return w_new[:R], m_new[:R]


# ---- duplication model (Sec. 4.2 "Using IKJTs") --------------------------------------------
def dedupe_len(l: float, B: float, S: float, d: float) -> float:
    """Expected size of the values slice after deduplicating a feature."""
    return l * B * (1.0 - (S - 1.0) / S * d)


def dedupe_factor(l: float, B: float, S: float, d: float) -> float:
    """Ratio of the original values slice length to the deduplicated one."""
    return l * B / dedupe_len(l, B, S, d)


def decode_ikjt(F: int, B: int, u_values, u_offsets, inverse, feat_uoff) -> List[List[List[int]]]:
    """Rebuild the per-row lists an IKJT encodes (Sec. 6.2: same logical data as the KJT)."""
    out = []
    for f in range(F):
        rows = []
        for b in range(B):
            u = int(feat_uoff[f]) + int(inverse[f * B + b])
            rows.append([int(x) for x in u_values[int(u_offsets[u]):int(u_offsets[u + 1])]])
        out.append(rows)
    return out
