"""Seeded synthetic inputs for DLRM-RMC style forward passes.

This module only *draws inputs*: table values, sparse ids, pooling lengths,
dense features and master MLP weights.  It holds none of the model's
arithmetic (no pooling, no matrix product, no interaction) so that both the
CPU oracle's tests and the GPU path's tests can be fed from it without
sharing any computation.

The workloads stand in for the production models of Table I (DLRM-RMC1/2/3:
about 10 or 100 embedding tables of 1M-20M rows, 20-160 or 20-50 lookups per
table with pooling, Bottom-FC / Predict-FC stacks; MT-WnD: 26 tables, one
lookup each, no Bottom-FC, N Predict-FC towers) and for the production
query traces of Sec. II-A (variable pooling factors, Fig. 2(c)); neither is
public, so shapes follow Table I and values are drawn here.

Two generators are used:

* Table values are *procedural*: element (t, r, d) is a pure function of
  (seed, t, r, d) built on the SplitMix64 output function (Steele, Lea,
  Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014):
  the n-th output of a SplitMix64 stream seeded with s is mix64(s + (n+1)*G)
  with G = 0x9e3779b97f4a7c15.  Any row can therefore be produced on demand,
  which is what lets a 150 GB table set be filled on the device while a CPU
  check materialises only the rows a few bags touch.
* Everything else comes from numpy's Philox bit generator keyed by
  (seed, stream id).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

MASTER_SEED = 2203

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# Table values are u24 * (0.05 * 2^-23) - 0.05, i.e. uniform on a 2^24-point
# grid of [-0.05, 0.05).  The scale is one fp32 constant so that a single
# IEEE multiply gives the same bits on every machine.
TABLE_HALF_RANGE = np.float32(0.05)
_TABLE_SCALE = np.float32(TABLE_HALF_RANGE * np.float32(2.0 ** -23))


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    num_tables: int
    rows: int                    # rows per table (all tables alike)
    emb_dim: int
    table_dtype: str             # "f32" | "f16"
    batch: int
    num_dense: int
    pooling: Tuple               # ("fixed", L) | ("poisson", mean, lo, hi)
    index_dist: Tuple            # ("uniform",) | ("zipf", alpha)
    bottom: Tuple[int, ...]      # widths F, ..., D; (F,) alone = no Bottom-FC
    top: Tuple[int, ...]         # widths interact_width, ..., 1
    seed: int = MASTER_SEED
    interaction: str = "dot"     # "dot": pairwise dots | "concat": plain concatenation
    towers: int = 1              # Predict-FC stacks (tasks), each of widths `top`

    @property
    def interact_width(self) -> int:
        t = self.num_tables
        if self.interaction == "concat":
            return self.bottom[-1] + t * self.emb_dim
        return self.emb_dim + t * (t + 1) // 2

    def with_batch(self, batch: int) -> "Workload":
        return replace(self, batch=batch)

    def with_uniform_indices(self) -> "Workload":
        return replace(self, index_dist=("uniform",), name=self.name + "-uniform")


def _tri(t: int, d: int) -> int:
    return d + t * (t + 1) // 2


WORKLOADS: Dict[str, Workload] = {
    # Tiny model a CPU check finishes in seconds.
    "tiny": Workload("tiny", 8, 100_000, 32, "f32", 256, 13, ("fixed", 20),
                     ("uniform",), (13, 256, 128, 32), (_tri(8, 32), 64, 1)),
    # RMC1-style, sparse-light (Table I row DLRM-RMC1).
    "rmc1": Workload("rmc1", 10, 4_000_000, 64, "f32", 1024, 256, ("fixed", 80),
                     ("zipf", 1.05), (256, 128, 64), (_tri(10, 64), 256, 64, 1)),
    # RMC2-style, sparse-heavy (Table I row DLRM-RMC2).
    "rmc2": Workload("rmc2", 40, 2_000_000, 64, "f16", 4096, 256,
                     ("poisson", 80.0, 1, 200), ("zipf", 1.05),
                     (256, 256, 64), (_tri(40, 64), 512, 128, 1)),
    # RMC3-style, dense-heavy (Table I row DLRM-RMC3).
    "rmc3": Workload("rmc3", 10, 1_000_000, 32, "f32", 4096, 2560, ("fixed", 20),
                     ("uniform",), (2560, 1024, 256, 32), (_tri(10, 32), 512, 256, 1)),
    # Large-capacity RMC2 variant: about 154 GB of fp16 rows.
    "rmc2-large": Workload("rmc2-large", 60, 20_000_000, 64, "f16", 4096, 256,
                           ("poisson", 80.0, 1, 200), ("zipf", 1.2),
                           (256, 256, 64), (_tri(60, 64), 512, 128, 1)),
    # MT-WnD-style (Table I row MT-WnD, "small" 1M-row tables): one lookup per
    # table, no pooling, no Bottom-FC, no interaction, 4 task towers.
    "mtwnd": Workload("mtwnd", 26, 1_000_000, 64, "f16", 4096, 64, ("fixed", 1),
                      ("zipf", 1.05), (64,), (64 + 26 * 64, 1024, 512, 256, 1),
                      interaction="concat", towers=4),
    # The same shape shrunk to what a CPU check finishes in seconds, with
    # ragged widths and a Bottom-FC layer.
    "mtwnd-tiny": Workload("mtwnd-tiny", 5, 50_000, 32, "f32", 200, 24, ("fixed", 1),
                           ("uniform",), (24, 40), (40 + 5 * 32, 96, 72, 1),
                           interaction="concat", towers=3),
}


# --------------------------------------------------------------------------
# procedural table values
# --------------------------------------------------------------------------
def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def table_counter(table: int, rows: np.ndarray, emb_dim: int) -> np.ndarray:
    """Counter n of element (table, row, col): ((table << 32) + row) * 1024 + col."""
    assert emb_dim <= 1024
    r = np.asarray(rows, dtype=np.uint64).reshape(-1, 1)
    c = np.arange(emb_dim, dtype=np.uint64).reshape(1, -1)
    return ((np.uint64(table) << np.uint64(32)) + r) * np.uint64(1024) + c


def table_rows(seed: int, table: int, rows: np.ndarray, emb_dim: int,
               dtype: str) -> np.ndarray:
    """Values of the given rows of one table, as stored ([len(rows), D])."""
    with np.errstate(over="ignore"):
        n = table_counter(table, rows, emb_dim)
        z = _mix64(np.uint64(seed) + (n + np.uint64(1)) * _GOLDEN)
    u24 = (z >> np.uint64(40)).astype(np.int64)
    v = (u24 - (1 << 23)).astype(np.float32) * _TABLE_SCALE
    if dtype == "f16":
        return v.astype(np.float16)        # round-to-nearest-even
    assert dtype == "f32"
    return v


def full_table(w: Workload, table: int) -> np.ndarray:
    """Whole table on the host; only sensible for small workloads."""
    out = np.empty((w.rows, w.emb_dim),
                   dtype=np.float16 if w.table_dtype == "f16" else np.float32)
    step = 1 << 18
    for lo in range(0, w.rows, step):
        hi = min(w.rows, lo + step)
        out[lo:hi] = table_rows(w.seed, table, np.arange(lo, hi), w.emb_dim,
                                w.table_dtype)
    return out


# --------------------------------------------------------------------------
# Philox sub-streams
# --------------------------------------------------------------------------
_STREAM_IDS = {"lengths": 1, "indices": 2, "dense": 3, "weights": 4, "perm": 5}


def _rng(seed: int, kind: str, a: int = 0, b: int = 0) -> np.random.Generator:
    sid = (_STREAM_IDS[kind] << 48) | ((a & 0xFFFFFF) << 24) | (b & 0xFFFFFF)
    return np.random.Generator(np.random.Philox(key=[seed, sid]))


# --------------------------------------------------------------------------
# sparse ids
# --------------------------------------------------------------------------
def zipf_cdf(rows: int, alpha: float) -> np.ndarray:
    """CDF of the bounded Zipf law P(k) = k^-alpha / H(rows, alpha), k = 1..rows."""
    p = np.arange(1, rows + 1, dtype=np.float64) ** (-alpha)
    c = np.cumsum(p)
    c /= c[-1]
    return c


def rank_permutation(seed: int, table: int, rows: int) -> Tuple[int, int]:
    """(a, c) of the bijection rank -> (a * rank + c) mod rows, gcd(a, rows) = 1.

    It scatters the popular ranks over the table so that popularity carries
    no spatial locality.
    """
    g = _rng(seed, "perm", table)
    a = int(g.integers(1, max(rows, 2)))
    while math.gcd(a, rows) != 1:      # a = 1 always qualifies, so this ends
        a = a + 1 if a + 1 < rows else 1
    c = int(g.integers(0, rows))
    return a, c


def draw_lengths(w: Workload, batch_id: int) -> np.ndarray:
    """Pooling lengths, int32 [T * B], table-major (entry t * B + b)."""
    n = w.num_tables * w.batch
    if w.pooling[0] == "fixed":
        return np.full(n, int(w.pooling[1]), dtype=np.int32)
    _, mean, lo, hi = w.pooling
    g = _rng(w.seed, "lengths", batch_id)
    return np.clip(g.poisson(mean, size=n), lo, hi).astype(np.int32)


def draw_indices(w: Workload, batch_id: int, lengths: np.ndarray,
                 cdf: Optional[np.ndarray] = None, workers: int = 1) -> np.ndarray:
    """Row ids, int32 [sum(lengths)], concatenated in the order of `lengths`.
    Every table has a stream of its own, so `workers` threads may draw the
    tables side by side; the result does not depend on their number."""
    per_table = lengths.reshape(w.num_tables, w.batch).sum(axis=1, dtype=np.int64)
    out = np.empty(int(per_table.sum()), dtype=np.int32)
    if w.index_dist[0] == "zipf" and cdf is None:
        cdf = zipf_cdf(w.rows, float(w.index_dist[1]))
    starts = np.concatenate([[0], np.cumsum(per_table)])

    def one_table(t: int) -> None:
        n = int(per_table[t])
        g = _rng(w.seed, "indices", batch_id, t)
        if w.index_dist[0] == "uniform":
            ids = g.integers(0, w.rows, size=n, dtype=np.int64)
        else:
            u = g.random(n)
            rank = np.minimum(np.searchsorted(cdf, u, side="right"), w.rows - 1)
            a, c = rank_permutation(w.seed, t, w.rows)
            ids = (rank.astype(np.int64) * a + c) % w.rows
        out[int(starts[t]):int(starts[t]) + n] = ids

    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(one_table, range(w.num_tables)))
    else:
        for t in range(w.num_tables):
            one_table(t)
    return out


def draw_dense(w: Workload, batch_id: int) -> np.ndarray:
    """Dense features ~ N(0, 1), float32 [B, F]."""
    g = _rng(w.seed, "dense", batch_id)
    return g.standard_normal((w.batch, w.num_dense), dtype=np.float32)


def draw_mlp(w: Workload, which: str, tower: int = 0) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Master fp32 weights [out, in] and biases [out], both ~ N(0, 1/fan_in)
    (variance 1/fan_in), for the "bottom" stack or tower `tower` of the "top" one."""
    widths = w.bottom if which == "bottom" else w.top
    base = 0 if which == "bottom" else 100
    layers = []
    for i in range(len(widths) - 1):
        fan_in, fan_out = widths[i], widths[i + 1]
        g = _rng(w.seed, "weights", base + i, tower)
        std = np.float32(fan_in ** -0.5)
        W = g.standard_normal((fan_out, fan_in), dtype=np.float32) * std
        b = g.standard_normal(fan_out, dtype=np.float32) * std
        layers.append((W, b))
    return layers


def profile_hot_rows(w: Workload, batch_ids, n_hot: int, cdf: Optional[np.ndarray] = None):
    """Per table, the n_hot row ids seen most often in the given (profiling)
    batches, most frequent first: a stand-in for ranking rows by access
    frequency over a production trace (Sec. IV-A).  Returns a list of int32 arrays."""
    counts = [np.zeros(w.rows, dtype=np.int32) for _ in range(w.num_tables)]
    for bid in batch_ids:
        lengths = draw_lengths(w, bid)
        ids = draw_indices(w, bid, lengths, cdf)
        per_table = lengths.reshape(w.num_tables, w.batch).sum(axis=1, dtype=np.int64)
        pos = 0
        for t in range(w.num_tables):
            n = int(per_table[t])
            counts[t] += np.bincount(ids[pos:pos + n], minlength=w.rows).astype(np.int32)
            pos += n
    out = []
    for t in range(w.num_tables):
        k = min(n_hot, w.rows)
        top = np.argpartition(counts[t], w.rows - k)[w.rows - k:]
        top = top[np.argsort(-counts[t][top], kind="stable")]
        out.append(top.astype(np.int32))
    return out


@dataclass
class Batch:
    dense: np.ndarray      # float32 [B, F]
    indices: np.ndarray    # int32 [nnz]
    lengths: np.ndarray    # int32 [T * B]
    nnz: int = field(init=False)

    def __post_init__(self):
        self.nnz = int(self.indices.shape[0])


def draw_batch(w: Workload, batch_id: int, cdf: Optional[np.ndarray] = None, workers: int = 1) -> Batch:
    lengths = draw_lengths(w, batch_id)
    return Batch(draw_dense(w, batch_id), draw_indices(w, batch_id, lengths, cdf, workers), lengths)


# --------------------------------------------------------------------------
# slicing a workload down to what a CPU check can hold
# --------------------------------------------------------------------------
def slice_samples(w: Workload, batch: Batch, samples: np.ndarray) -> Batch:
    """The sub-batch made of the given sample positions (in that order)."""
    T, B = w.num_tables, w.batch
    samples = np.asarray(samples, dtype=np.int64)
    off = np.zeros(T * B + 1, dtype=np.int64)
    np.cumsum(batch.lengths, out=off[1:])
    len2d = batch.lengths.reshape(T, B)
    new_len = len2d[:, samples].reshape(-1).astype(np.int32)
    parts = []
    for t in range(T):
        for b in samples:
            k = t * B + int(b)
            parts.append(batch.indices[off[k]:off[k + 1]])
    idx = np.concatenate(parts) if parts else np.empty(0, np.int32)
    return Batch(batch.dense[samples].copy(), idx.astype(np.int32), new_len)


def compact_tables(w: Workload, batch: Batch, n_samples: int):
    """Materialise only the rows a batch touches.

    Returns (tables, indices) where tables[t] is [n_unique_t, D] in storage
    dtype and `indices` addresses those compact tables; bags and their order
    are unchanged, so any function of the gathered rows is unchanged too.
    """
    T = w.num_tables
    per_table = batch.lengths.reshape(T, n_samples).sum(axis=1, dtype=np.int64)
    new_idx = np.empty_like(batch.indices)
    tables = []
    pos = 0
    for t in range(T):
        n = int(per_table[t])
        ids = batch.indices[pos:pos + n]
        uniq, inv = np.unique(ids, return_inverse=True)
        tables.append(table_rows(w.seed, t, uniq, w.emb_dim, w.table_dtype))
        new_idx[pos:pos + n] = inv.astype(np.int32)
        pos += n
    return tables, new_idx
