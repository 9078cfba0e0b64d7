"""Seeded synthetic inputs for the sparse/dense gradient aggregation path.

This module only *draws* inputs: row ids, value rows, embedding tables and dense
gradient buffers.  It contains none of the aggregation, partitioning or
optimizer arithmetic, so both the CPU oracle's tests and the HIP path's tests
may use it without sharing any of the method's code.

The paper's sparse workloads are an 800K-word, 512-wide language-model
embedding and 1024-wide translation embeddings, trained with 48 workers at a
batch of 128 sequences per worker (Sec. 6.1).  Their corpora are not available
here, so ids are drawn from a bounded Zipf law over a frequency-ranked
vocabulary (id = rank - 1) and values from N(0, 1); only the shapes come from
the paper.

Everything is generated on the host with ``numpy.random.Generator(PCG64)``.
Seed of a stream = BASE_SEED + 100 * workload.index + stream number, where the
stream numbers are ids 0, values 1, table 2, dense 3, id permutation 4, and a
second table adds 10.  Each worker's slice comes from its own child stream
(``SeedSequence(seed).spawn``), so workers can be generated independently and
in any order.
"""

from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 18080262100

STREAM_IDS = 0
STREAM_VALUES = 1
STREAM_TABLE = 2
STREAM_DENSE = 3
STREAM_PERMUTATION = 4
SECOND_TABLE = 10

TABLE_INIT_STD = 0.02


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic configuration: a sparse variable (or two) plus a dense part."""

    name: str
    index: int                  # selects the seed block
    vocab: int                  # V: rows of the embedding table
    dim: int                    # D: row width in elements
    n_workers: int              # N: simulated gradient sources
    n_per_worker: int           # n_w: ids per worker per table
    zipf_s: Optional[float]     # None -> uniform ids
    val_dtype: str              # "f32" or "bf16" (value rows as handed to the path)
    n_shards: int               # P
    hash: str                   # "mod" or "mul"
    optimizer: str              # "sgd" or "adagrad"
    lr: float
    accum_init: float           # Adagrad accumulator start value
    n_tables: int               # independent sparse variables
    dense_count: int            # C: elements per dense buffer (0 = no dense part)
    dense_dtype: str            # "f32" or "bf16"

    @property
    def total_rows(self) -> int:
        """M: input rows per table."""
        return self.n_workers * self.n_per_worker


TINY = Workload("tiny", 0, 10_000, 64, 4, 256, 1.0, "f32", 2, "mod",
                "sgd", 0.1, 0.1, 1, 65_536, "f32")
SMALL_LM = Workload("small_lm", 1, 100_000, 256, 8, 2_560, 1.1, "f32", 4, "mul",
                    "sgd", 0.05, 0.1, 1, 1 << 22, "f32")
LARGE_LM = Workload("large_vocab_lm", 2, 800_000, 512, 48, 2_560, 1.0, "f32", 8, "mul",
                    "adagrad", 0.2, 0.1, 1, 1 << 23, "f32")
NMT = Workload("nmt_like", 3, 32_768, 1_024, 48, 4_096, 1.2, "bf16", 8, "mul",
               "sgd", 1.0, 0.1, 2, 1 << 26, "bf16")
STRESS_UNIFORM = Workload("stress_uniform", 4, 4_000_000, 128, 64, 16_384, None, "f32", 16,
                          "mul", "adagrad", 0.1, 0.1, 1, 0, "f32")
STRESS_ZIPF = Workload("stress_zipf", 5, 4_000_000, 128, 64, 16_384, 1.3, "f32", 16,
                       "mul", "adagrad", 0.1, 0.1, 1, 0, "f32")

WORKLOADS = {w.name: w for w in
             (TINY, SMALL_LM, LARGE_LM, NMT, STRESS_UNIFORM, STRESS_ZIPF)}


def shrink(w: Workload, *, vocab: Optional[int] = None, n_workers: Optional[int] = None,
           n_per_worker: Optional[int] = None, dim: Optional[int] = None,
           dense_count: Optional[int] = None) -> Workload:
    """Same recipe at a smaller size (for parity cases the oracle finishes in seconds)."""
    return dataclasses.replace(
        w,
        name=w.name + "_shrunk",
        vocab=w.vocab if vocab is None else vocab,
        n_workers=w.n_workers if n_workers is None else n_workers,
        n_per_worker=w.n_per_worker if n_per_worker is None else n_per_worker,
        dim=w.dim if dim is None else dim,
        dense_count=w.dense_count if dense_count is None else dense_count,
    )


def _seed(w: Workload, stream: int, table: int = 0) -> int:
    return BASE_SEED + 100 * w.index + stream + SECOND_TABLE * table


def _worker_rngs(seed: int, n: int) -> List[np.random.Generator]:
    return [np.random.Generator(np.random.PCG64(s))
            for s in np.random.SeedSequence(seed).spawn(n)]


# ---------------------------------------------------------------- bf16 storage

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even; NaN stays NaN); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    rounded = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    return np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16), rounded)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------------------- ids

def zipf_cdf(vocab: int, s: float) -> np.ndarray:
    """Cumulative weights of p(k) ~ k**-s, k = 1..vocab, normalised, float64."""
    wts = np.arange(1, vocab + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(wts)
    cdf /= cdf[-1]
    return cdf


def draw_ids(rng: np.random.Generator, vocab: int, s: Optional[float], n: int,
             cdf: Optional[np.ndarray] = None) -> np.ndarray:
    """n int64 ids in [0, vocab): bounded Zipf by inverse CDF (id = rank - 1), or uniform."""
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    if s is None:
        return rng.integers(0, vocab, size=n, dtype=np.int64)
    if cdf is None:
        cdf = zipf_cdf(vocab, s)
    u = rng.random(n)
    ids = np.searchsorted(cdf, u, side="left").astype(np.int64)
    np.minimum(ids, vocab - 1, out=ids)
    return ids


def id_permutation(w: Workload, table: int = 0) -> np.ndarray:
    """A fixed random relabelling of [0, vocab), to scatter the hot ids over the table."""
    rng = np.random.Generator(np.random.PCG64(_seed(w, STREAM_PERMUTATION, table)))
    return rng.permutation(w.vocab).astype(np.int64)


def sparse_ids(w: Workload, table: int = 0, permute: bool = False) -> List[np.ndarray]:
    """Per-worker int64 id arrays of one sparse variable."""
    rngs = _worker_rngs(_seed(w, STREAM_IDS, table), w.n_workers)
    cdf = None if w.zipf_s is None else zipf_cdf(w.vocab, w.zipf_s)
    out = [draw_ids(r, w.vocab, w.zipf_s, w.n_per_worker, cdf) for r in rngs]
    if permute:
        perm = id_permutation(w, table)
        out = [perm[i] for i in out]
    return out


# ---------------------------------------------------------------------- values

def normal_f32(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def sparse_values(w: Workload, table: int = 0) -> List[np.ndarray]:
    """Per-worker value rows [n_w, D]: float32, or uint16 bf16 patterns when val_dtype is bf16."""
    rngs = _worker_rngs(_seed(w, STREAM_VALUES, table), w.n_workers)
    out = []
    for r in rngs:
        v = normal_f32(r, (w.n_per_worker, w.dim))
        out.append(f32_to_bf16_bits(v) if w.val_dtype == "bf16" else v)
    return out


def small_integer_values(rng: np.random.Generator, shape, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Integer-valued float32 rows: every partial sum is exact, whatever the order."""
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def table_init(w: Workload, table: int = 0) -> np.ndarray:
    """Embedding table [V, D] float32, N(0, 0.02**2)."""
    rng = np.random.Generator(np.random.PCG64(_seed(w, STREAM_TABLE, table)))
    t = normal_f32(rng, (w.vocab, w.dim))
    t *= np.float32(TABLE_INIT_STD)
    return t


def accum_init(w: Workload) -> np.ndarray:
    """Adagrad accumulator [V, D] float32, constant start value."""
    return np.full((w.vocab, w.dim), w.accum_init, dtype=np.float32)


def dense_rngs(w: Workload) -> List[np.random.Generator]:
    return _worker_rngs(_seed(w, STREAM_DENSE), w.n_workers)


def dense_buffer(w: Workload, rng: np.random.Generator, count: Optional[int] = None) -> np.ndarray:
    """One worker's dense gradient buffer: float32 N(0,1), or bf16 patterns (uint16)."""
    c = w.dense_count if count is None else count
    v = normal_f32(rng, (c,))
    return f32_to_bf16_bits(v) if w.dense_dtype == "bf16" else v


def dense_buffers(w: Workload) -> List[np.ndarray]:
    return [dense_buffer(w, r) for r in dense_rngs(w)]


# ------------------------------------------------------------------ statistics

def id_statistics(ids: List[np.ndarray], vocab: int) -> Tuple[int, int, int, float]:
    """(M, U, longest run, mean per-worker fraction of the table touched)."""
    allids = np.concatenate(ids) if ids else np.zeros(0, np.int64)
    if allids.size == 0:
        return 0, 0, 0, 0.0
    uniq, cnt = np.unique(allids, return_counts=True)
    alpha = float(np.mean([np.unique(i).size for i in ids])) / float(vocab)
    return int(allids.size), int(uniq.size), int(cnt.max()), alpha
