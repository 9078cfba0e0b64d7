"""CPU oracle of the sparse/dense gradient aggregation path (arXiv 1808.02621).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path never routes
through it.  It shares no code with the HIP library and imports nothing from
the product package.

``px_oracle.cpp`` is the oracle itself (an ordered-map row accumulator in
double precision, scalar optimizer updates, a scalar mean); this file only
builds it with g++, loads it with ctypes and marshals numpy arrays.

Pins (tests/test_oracle_*.py): brute-force densification on tiny inputs,
column-sum / set-size / disjointness invariants, special cases that are
bit-exact, integer-valued inputs whose sums are order independent, the first
Adagrad step's closed form, PyTorch's CPU sparse-coalesce and sparse
optimizer routines, and numpy's fancy indexing for the lookup.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "px_oracle.cpp")
LIBRARY = os.path.join(_HERE, "libpx_oracle.so")

DT_F32, DT_BF16 = 0, 1
HASH_MOD, HASH_MUL = 0, 1
AGG_SUM, AGG_AVERAGE = 0, 1

_lib = None


SANITIZE_FLAGS = ("-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=all")


def build(source: str = SOURCE, output: str = LIBRARY, extra_flags: Sequence[str] = ()) -> str:
    """Compile the oracle with g++ (always recompiles).  extra_flags, e.g. SANITIZE_FLAGS, come
    after -O2 and so override it."""
    cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Wextra", *extra_flags,
           "-o", output, source]
    subprocess.run(cmd, check=True)
    return output


def _declare(lib) -> None:
    c_i64p = ctypes.POINTER(ctypes.c_int64)
    c_pp = ctypes.POINTER(ctypes.c_void_p)
    lib.pxo_sparse_coalesce.restype = ctypes.c_int64
    lib.pxo_sparse_coalesce.argtypes = [
        ctypes.c_int, c_pp, c_pp, c_i64p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
        ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.pxo_partition_rows.restype = ctypes.c_int
    lib.pxo_partition_rows.argtypes = [
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_void_p]
    lib.pxo_sparse_apply_sgd.restype = ctypes.c_int
    lib.pxo_sparse_apply_sgd.argtypes = [
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int64, ctypes.c_void_p, ctypes.c_double]
    lib.pxo_sparse_apply_adagrad.restype = ctypes.c_int
    lib.pxo_sparse_apply_adagrad.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_double]
    lib.pxo_sparse_lookup.restype = ctypes.c_int
    lib.pxo_sparse_lookup.argtypes = [
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
    lib.pxo_dense_average.restype = ctypes.c_int
    lib.pxo_dense_average.argtypes = [
        ctypes.c_int, c_pp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]


def load(path: Optional[str] = None):
    """Load the oracle library (building it first if it was never built)."""
    global _lib
    if path is not None:
        lib = ctypes.CDLL(path)
        _declare(lib)
        return lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            build()
        _lib = ctypes.CDLL(LIBRARY)
        _declare(_lib)
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DT_F32
    if a.dtype == np.uint16:          # bfloat16 bit patterns
        return DT_BF16
    raise TypeError("values must be float32 or uint16 (bfloat16 patterns), got %s" % a.dtype)


def _ptr_array(arrays: Sequence[np.ndarray]):
    return (ctypes.c_void_p * max(1, len(arrays)))(*[a.ctypes.data for a in arrays])


class RepeatedId(ValueError):
    pass


class IdOutOfRange(ValueError):
    pass


def sparse_coalesce(idx: Sequence[np.ndarray], val: Sequence[np.ndarray], dim: int, vocab: int,
                    average: bool = False, lib=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(ids ascending [U] int64, rows [U, dim] float32, run_len [U] int32)."""
    lib = lib or load()
    n = len(idx)
    assert len(val) == n
    idx = [np.ascontiguousarray(i, dtype=np.int64) for i in idx]
    val = [np.ascontiguousarray(v) for v in val]
    code = _dtype_code(val[0]) if n else DT_F32
    for i, v in zip(idx, val):
        assert _dtype_code(v) == code and v.size == i.size * dim
    counts = np.array([i.size for i in idx], dtype=np.int64)
    m = int(counts.sum())
    out_ids = np.empty(m, dtype=np.int64)
    out_rows = np.empty((m, dim), dtype=np.float32)
    out_len = np.empty(m, dtype=np.int32)
    u = lib.pxo_sparse_coalesce(
        n, _ptr_array(idx), _ptr_array(val),
        counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), dim, code, vocab,
        AGG_AVERAGE if average else AGG_SUM, out_ids.ctypes.data, out_rows.ctypes.data,
        out_len.ctypes.data)
    if u < 0:
        raise IdOutOfRange("an id lies outside [0, %d)" % vocab)
    return out_ids[:u].copy(), out_rows[:u].copy(), out_len[:u].copy()


def partition_rows(ids: np.ndarray, n_shards: int, hash: str = "mul", lib=None
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(shard [n] int32, perm [n] int32, offsets [P+1] int64)."""
    lib = lib or load()
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    n = ids.size
    shard = np.empty(n, dtype=np.int32)
    perm = np.empty(n, dtype=np.int32)
    offsets = np.empty(n_shards + 1, dtype=np.int64)
    rc = lib.pxo_partition_rows(ids.ctypes.data, n, n_shards,
                                HASH_MUL if hash == "mul" else HASH_MOD,
                                shard.ctypes.data, perm.ctypes.data, offsets.ctypes.data)
    if rc:
        raise ValueError("bad shard count")
    return shard, perm, offsets


def _check_apply(rc: int) -> None:
    if rc == 2:
        raise IdOutOfRange("an id lies outside the table")
    if rc == 4:
        raise RepeatedId("apply needs distinct ids")
    if rc:
        raise ValueError("oracle apply failed: %d" % rc)


def sparse_apply_sgd(table: np.ndarray, ids: np.ndarray, rows: np.ndarray, lr: float,
                     perm: Optional[np.ndarray] = None, lib=None) -> None:
    """In place on ``table`` ([V, D] float32, C-contiguous)."""
    lib = lib or load()
    assert table.dtype == np.float32 and table.flags.c_contiguous and table.flags.writeable
    vocab, dim = table.shape
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    assert rows.size == ids.size * dim
    p = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    _check_apply(lib.pxo_sparse_apply_sgd(
        table.ctypes.data, vocab, dim, ids.ctypes.data, rows.ctypes.data, ids.size,
        None if p is None else p.ctypes.data, float(lr)))


def sparse_apply_adagrad(table: np.ndarray, accum: np.ndarray, ids: np.ndarray, rows: np.ndarray,
                         lr: float, eps: float = 0.0, perm: Optional[np.ndarray] = None,
                         lib=None) -> None:
    """In place on ``table`` and ``accum`` (both [V, D] float32, C-contiguous)."""
    lib = lib or load()
    for t in (table, accum):
        assert t.dtype == np.float32 and t.flags.c_contiguous and t.flags.writeable
    assert table.shape == accum.shape
    vocab, dim = table.shape
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    assert rows.size == ids.size * dim
    p = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    _check_apply(lib.pxo_sparse_apply_adagrad(
        table.ctypes.data, accum.ctypes.data, vocab, dim, ids.ctypes.data, rows.ctypes.data,
        ids.size, None if p is None else p.ctypes.data, float(lr), float(eps)))


def sparse_lookup(table: np.ndarray, ids: np.ndarray, perm: Optional[np.ndarray] = None,
                  first: int = 0, last: Optional[int] = None, out: Optional[np.ndarray] = None,
                  lib=None) -> np.ndarray:
    """out[k] = table[ids[k]] for k = perm[j], j in [first, last); other rows of out are kept."""
    lib = lib or load()
    assert table.dtype == np.float32 and table.flags.c_contiguous
    vocab, dim = table.shape
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    n = ids.size
    if out is None:
        out = np.zeros((n, dim), dtype=np.float32)
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.shape == (n, dim)
    p = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    rc = lib.pxo_sparse_lookup(table.ctypes.data, vocab, dim, ids.ctypes.data, n,
                               None if p is None else p.ctypes.data, first, n if last is None else last,
                               out.ctypes.data)
    if rc == 2:
        raise IdOutOfRange("an id lies outside the table")
    return out


def dense_average(bufs: Sequence[np.ndarray], average: bool = True, lib=None) -> np.ndarray:
    """Element-wise sum (or mean over the buffers) of N equal-length buffers, float32."""
    lib = lib or load()
    bufs = [np.ascontiguousarray(b) for b in bufs]
    assert bufs, "need at least one buffer"
    code = _dtype_code(bufs[0])
    count = bufs[0].size
    for b in bufs:
        assert _dtype_code(b) == code and b.size == count
    out = np.empty(count, dtype=np.float32)
    lib.pxo_dense_average(len(bufs), _ptr_array(bufs), count, code,
                          AGG_AVERAGE if average else AGG_SUM, out.ctypes.data)
    return out
