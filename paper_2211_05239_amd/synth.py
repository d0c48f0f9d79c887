"""Seeded synthetic session-structured KJT batches (input generation only).

This module draws the *inputs* of the deduplication path: session sizes, per-session base
lists, per-sample redraws, embedding tables and upstream gradients.  It holds none of the
method's arithmetic (no hashing, no deduplication, no pooling) and is the only code shared
by the CPU oracle's tests and the HIP path's tests/benchmarks.

The batches stand in for the session-clustered production batches the paper trains on
(Sec. 3: a session's samples are adjacent after clustering and mostly repeat the same
sparse-feature lists; Sec. 4.2: d(f) is the probability that a feature keeps its value
between adjacent rows of a session).

Layout produced (feature-major KJT, Sec. 4.2):
  values  int64 [N]        ids of feature 0's rows 0..B-1, then feature 1's rows, ...
  offsets int64 [F*B + 1]  offsets[f*B + b] = start of row b of feature f in `values`;
                           one trailing sentinel offsets[F*B] = N.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20221105


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the configuration list (1-based), used in the seed
    B: int                # samples per batch
    F: int                # sparse features (= embedding tables)
    S: float              # mean session size
    len_law: str          # "uniform" | "zipf"
    len_max: int          # uniform: 0..len_max ; zipf: 1..len_max
    len_a: float          # zipf exponent for lengths
    id_law: str           # "uniform" | "zipf"
    id_a: float           # zipf exponent for ids
    rows: int             # rows per table
    D: int                # embedding dimension
    table_dtype: str      # "f32" | "f16" | "bf16"
    redraw: float = 0.0   # probability that a non-first sample of a session redraws all features
    shift: float = 0.0    # probability that a non-first sample's list is the previous one shifted by
                          # one id (oldest id dropped, a new id appended), drawn per feature


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("cfg1", 1, 512, 4, 4, "uniform", 20, 0.0, "uniform", 0.0, 100_000, 64, "f32"),
        Workload("cfg2", 2, 4096, 16, 8, "zipf", 100, 1.2, "zipf", 1.05, 1_000_000, 128, "f32", 0.1),
        Workload("cfg3", 3, 16384, 64, 16, "zipf", 256, 1.1, "zipf", 1.05, 1_000_000, 128, "f16"),
        Workload("cfg4", 4, 8192, 32, 8, "uniform", 128, 0.0, "uniform", 0.0, 1_000_000, 128, "f32"),
        Workload("cfg5", 5, 16384, 64, 16, "zipf", 256, 1.1, "zipf", 1.05, 1_000_000, 128, "f32"),
    ]
}

SWEEP_SESSION_SIZES = (1, 2, 4, 8, 32)


def sweep_workload(S: float) -> Workload:
    """Duplication-sweep member: cfg4 with mean session size S."""
    return dataclasses.replace(WORKLOADS["cfg4"], name=f"cfg4_S{int(S)}", S=float(S))


def scaled(w: Workload, **kw) -> Workload:
    """A smaller copy of a workload (same laws, other sizes) for CPU-sized tests."""
    return dataclasses.replace(w, **kw)


@dataclasses.dataclass
class Batch:
    F: int
    B: int
    values: np.ndarray        # int64 [N]
    offsets: np.ndarray       # int64 [F*B+1]
    session_of: np.ndarray    # int32 [B] session number of each sample
    mean_session: float

    @property
    def N(self) -> int:
        return int(self.values.shape[0])


def _zipf_cdf(n: int, a: float) -> np.ndarray:
    k = np.arange(1, n + 1, dtype=np.float64)
    p = k ** (-a)
    c = np.cumsum(p)
    return c / c[-1]


_CDF_CACHE: Dict[tuple, np.ndarray] = {}


def _bounded_zipf(rng: np.random.Generator, n_draws: int, n: int, a: float) -> np.ndarray:
    """Ranks in 1..n with P(k) proportional to k**-a (inverse-CDF table lookup)."""
    key = (n, a)
    cdf = _CDF_CACHE.get(key)
    if cdf is None:
        cdf = _zipf_cdf(n, a)
        _CDF_CACHE[key] = cdf
    u = rng.random(n_draws)
    k = np.searchsorted(cdf, u, side="right")
    return np.minimum(k, n - 1).astype(np.int64) + 1


def _draw_lengths(rng, w: Workload, n: int) -> np.ndarray:
    if w.len_law == "uniform":
        return rng.integers(0, w.len_max + 1, size=n, dtype=np.int64)
    return _bounded_zipf(rng, n, w.len_max, w.len_a)


def _draw_ids(rng, w: Workload, n: int) -> np.ndarray:
    if w.id_law == "uniform":
        return rng.integers(0, w.rows, size=n, dtype=np.int64)
    return _bounded_zipf(rng, n, w.rows, w.id_a) - 1


def _session_layout(rng, B: int, S: float):
    """Contiguous sessions with Geometric(1/S) sizes on {1,2,...}; the last one is cut at B."""
    if S <= 1.0:
        sizes = np.ones(B, dtype=np.int64)
    else:
        sizes = np.zeros(0, dtype=np.int64)
        while sizes.sum() < B:
            sizes = np.concatenate([sizes, rng.geometric(1.0 / S, size=max(16, int(2 * B / S)))])
        cut = int(np.searchsorted(np.cumsum(sizes), B, side="left")) + 1
        sizes = sizes[:cut].copy()
        sizes[-1] -= sizes.sum() - B
    starts = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    session_of = np.repeat(np.arange(len(sizes), dtype=np.int32), sizes)
    first_of = np.repeat(starts, sizes)  # first sample of my session
    return sizes, session_of, first_of


def make_batch(w: Workload, batch_index: int = 0, seed: Optional[int] = None) -> Batch:
    """One seeded batch. seed defaults to BASE_SEED + 1000*w.index + batch_index."""
    if seed is None:
        seed = BASE_SEED + 1000 * w.index + batch_index
    rng = np.random.default_rng(seed)
    B, F = w.B, w.F
    sizes, session_of, first_of = _session_layout(rng, B, w.S)

    # src[b] = the sample whose draw sample b carries: the session's first sample, or b itself
    # when b is a "changed" sample that redraws every feature.
    src = first_of.copy()
    if w.redraw > 0.0:
        changed = (rng.random(B) < w.redraw) & (np.arange(B) != first_of)
        src[changed] = np.arange(B)[changed]
    draw_ids_of_sample, draw_index = np.unique(src, return_inverse=True)
    K = len(draw_ids_of_sample)

    vals, offs = [], [np.zeros(1, dtype=np.int64)]
    base = 0
    if w.shift > 0.0:
        assert w.redraw == 0.0, "shifted lists are generated for sessions without redraws"
    for _f in range(F):
        dl = _draw_lengths(rng, w, K)
        if w.shift > 0.0:
            # A session's samples are windows sliding over one id stream: a shifted sample starts one
            # id later than its predecessor and keeps the session's list length.
            moved = (rng.random(B) < w.shift) & (np.arange(B) != first_of)
            cs = np.cumsum(moved)
            sigma = (cs - cs[first_of]) * (dl[draw_index] > 0)   # shifts since the session's start
            last_of = np.concatenate([first_of[1:][np.diff(first_of) != 0] - 1, [B - 1]])
            stream = dl + sigma[last_of] * (dl > 0)
        else:
            sigma = 0
            stream = dl
        doff = np.concatenate([[0], np.cumsum(stream)])
        dids = _draw_ids(rng, w, int(doff[-1]))
        sl = dl[draw_index]                        # per-sample length
        soff = np.concatenate([[0], np.cumsum(sl)])
        n_f = int(soff[-1])
        gather = np.repeat(doff[draw_index] + sigma - soff[:-1], sl) + np.arange(n_f, dtype=np.int64)
        vals.append(dids[gather])
        offs.append(soff[1:] + base)
        base += n_f
    values = np.concatenate(vals) if vals else np.zeros(0, dtype=np.int64)
    offsets = np.concatenate(offs).astype(np.int64)
    return Batch(F, B, np.ascontiguousarray(values, dtype=np.int64), offsets, session_of,
                 float(B) / float(len(sizes)))


def make_tables(w: Workload, seed: Optional[int] = None, F: Optional[int] = None):
    """Host tables: F arrays [rows, D], N(0, std 0.01) drawn in fp32, then cast (RNE) to the
    table dtype.  bf16 is returned as uint16 bit patterns (numpy has no bfloat16)."""
    if seed is None:
        seed = BASE_SEED + 1000 * w.index + 777
    rng = np.random.default_rng(seed)
    out = []
    for _f in range(w.F if F is None else F):
        t = (rng.standard_normal((w.rows, w.D), dtype=np.float32) * np.float32(0.01))
        if w.table_dtype == "f16":
            t = t.astype(np.float16)
        elif w.table_dtype == "bf16":
            t = f32_to_bf16_bits(t)
        out.append(np.ascontiguousarray(t))
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Input formatting only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def make_grad_out(w: Workload, batch_index: int = 0, seed: Optional[int] = None) -> np.ndarray:
    """Upstream gradient of the expanded output, fp32 [F, B, D], N(0,1)*1e-2."""
    if seed is None:
        seed = BASE_SEED + 1000 * w.index + 500 + batch_index
    rng = np.random.default_rng(seed)
    return rng.standard_normal((w.F, w.B, w.D), dtype=np.float32) * np.float32(0.01)


def make_weights(batch: "Batch", seed: int = 0, perturb: float = 0.0) -> np.ndarray:
    """Per-id weights, fp32 [N], beside batch.values: one of eight levels 0.25 .. 2.0 chosen by the
    id, its position in the list and the seed, so rows that hold the same list hold the same weights
    (the duplication of the batch is kept).  With probability `perturb` a non-empty row gets another
    level on its first id: such a row differs from its copies in the weights only."""
    N = batch.values.shape[0]
    lens = np.diff(batch.offsets)
    pos = np.arange(N, dtype=np.int64) - np.repeat(batch.offsets[:-1], lens)
    level = (batch.values * 2654435761 + pos * 40503 + seed) % 8
    if perturb > 0.0:
        rng = np.random.default_rng(BASE_SEED + 77 + seed)
        hit = (rng.random(lens.shape[0]) < perturb) & (lens > 0)
        first = batch.offsets[:-1][hit]
        level[first] = (level[first] + 1 + rng.integers(0, 7, size=first.shape[0])) % 8
    return ((level + 1).astype(np.float32) * np.float32(0.25))


def tiny_batch(rng: np.random.Generator, F: int, B: int, alphabet: int, max_len: int) -> Batch:
    """Small-alphabet batch where lists coincide by content often (brute-force test food)."""
    vals, offs, base = [], [np.zeros(1, dtype=np.int64)], 0
    for _f in range(F):
        ln = rng.integers(0, max_len + 1, size=B, dtype=np.int64)
        off = np.cumsum(ln)
        vals.append(rng.integers(0, alphabet, size=int(off[-1]) if B else 0, dtype=np.int64))
        offs.append(off + base)
        base += int(off[-1]) if B else 0
    values = np.concatenate(vals) if vals else np.zeros(0, dtype=np.int64)
    return Batch(F, B, values.astype(np.int64), np.concatenate(offs).astype(np.int64),
                 np.arange(B, dtype=np.int32), 1.0)


def batch_from_lists(lists_per_feature) -> Batch:
    """Build a KJT from explicit python lists: lists_per_feature[f][b] is a list of ids."""
    F = len(lists_per_feature)
    B = len(lists_per_feature[0]) if F else 0
    vals, offs = [], [0]
    for f in range(F):
        assert len(lists_per_feature[f]) == B
        for b in range(B):
            vals.extend(int(x) for x in lists_per_feature[f][b])
            offs.append(len(vals))
    return Batch(F, B, np.asarray(vals, dtype=np.int64), np.asarray(offs, dtype=np.int64),
                 np.arange(B, dtype=np.int32), 1.0)
