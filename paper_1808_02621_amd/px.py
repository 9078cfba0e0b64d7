"""ctypes binding of libpx (include/px.h): argument marshalling only.

Every function has the name and meaning of the C entry point it calls; every
step of the path runs inside the HIP library.  PyTorch tensors are used as
device buffers and for the current stream, nothing else.  There is no
fallback: if the library is not built, importing this module raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PX_LIBRARY may name another build of the same library (e.g. one compiled with other tuning macros).
LIBRARY = os.environ.get("PX_LIBRARY") or os.path.join(_HERE, "libpx.so")

PX_OK = 0
PX_ERR_INVALID_ARG = 1
PX_ERR_INDEX_OUT_OF_RANGE = 2
PX_ERR_SCRATCH_TOO_SMALL = 3
PX_ERR_NOT_UNIQUE = 4
PX_ERR_DEVICE = 5

PX_F32, PX_BF16 = 0, 1
PX_HASH_MOD, PX_HASH_MUL = 0, 1
PX_MAX_SOURCES = 1024
PX_MAX_SHARDS = 256
PX_PARTITION_NOALLOC_MAX_IDS = 1 << 22

EXPORTS = [
    "px_create", "px_destroy", "px_status_string", "px_last_error", "px_device_status",
    "px_coalesce_scratch_bytes", "px_partition_scratch_bytes", "px_sparse_coalesce",
    "px_partition_rows", "px_sparse_apply_sgd", "px_sparse_apply_adagrad", "px_dense_average",
    "px_sparse_coalesce_apply_sgd", "px_sparse_coalesce_apply_adagrad", "px_sparse_lookup",
    "px_partition_cost_fit", "px_partition_cost_argmin", "px_partition_search_next",
    "px_dense_average_launches", "px_partition_rows_noalloc", "px_set_wait_limit",
]

if not os.path.exists(LIBRARY):
    raise ImportError(
        "%s is missing: build it with `python -m paper_1808_02621_amd.build` "
        "(there is no CPU or PyTorch fallback)" % LIBRARY)

lib = ctypes.CDLL(LIBRARY)

_vp, _i64, _int, _f32, _sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float,
                              ctypes.c_size_t)
_pp = ctypes.POINTER(ctypes.c_void_p)
_i64p = ctypes.POINTER(ctypes.c_int64)

lib.px_create.restype = _int
lib.px_create.argtypes = [ctypes.POINTER(_vp), _int]
lib.px_destroy.restype = _int
lib.px_destroy.argtypes = [_vp]
lib.px_status_string.restype = ctypes.c_char_p
lib.px_status_string.argtypes = [_int]
lib.px_last_error.restype = ctypes.c_char_p
lib.px_last_error.argtypes = [_vp]
lib.px_device_status.restype = _int
lib.px_device_status.argtypes = [_vp, _vp]
lib.px_set_wait_limit.restype = _int
lib.px_set_wait_limit.argtypes = [_vp, _i64]
lib.px_coalesce_scratch_bytes.restype = _sz
lib.px_coalesce_scratch_bytes.argtypes = [_i64, _i64]
lib.px_partition_scratch_bytes.restype = _sz
lib.px_partition_scratch_bytes.argtypes = [_i64]
lib.px_sparse_coalesce.restype = _int
lib.px_sparse_coalesce.argtypes = [_vp, _int, _pp, _pp, _i64p, _i64, _int, _i64, _f32, _vp, _vp, _vp,
                                   _vp, _vp, _sz, _vp]
lib.px_sparse_coalesce_apply_sgd.restype = _int
lib.px_sparse_coalesce_apply_sgd.argtypes = [_vp, _int, _pp, _pp, _i64p, _i64, _int, _i64, _f32, _vp, _f32, _vp,
                                             _vp, _vp, _vp, _sz, _vp]
lib.px_sparse_coalesce_apply_adagrad.restype = _int
lib.px_sparse_coalesce_apply_adagrad.argtypes = [_vp, _int, _pp, _pp, _i64p, _i64, _int, _i64, _f32, _vp, _vp,
                                                 _f32, _f32, _vp, _vp, _vp, _vp, _sz, _vp]
lib.px_sparse_lookup.restype = _int
lib.px_sparse_lookup.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _vp]
lib.px_partition_rows.restype = _int
lib.px_partition_rows.argtypes = [_vp, _vp, _vp, _i64, _int, _int, _vp, _vp, _vp, _vp, _sz, _vp]
lib.px_partition_rows_noalloc.restype = _int
lib.px_partition_rows_noalloc.argtypes = [_vp, _vp, _vp, _i64, _int, _int, _vp, _vp, _vp, _vp]
lib.px_sparse_apply_sgd.restype = _int
lib.px_sparse_apply_sgd.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _f32, _vp]
lib.px_sparse_apply_adagrad.restype = _int
lib.px_sparse_apply_adagrad.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _f32,
                                        _f32, _vp]
lib.px_dense_average.restype = _int
lib.px_dense_average.argtypes = [_vp, _int, _pp, _i64, _int, _vp, _int, _f32, _vp]
lib.px_dense_average_launches.restype = _i64
lib.px_dense_average_launches.argtypes = [_int, _i64, _int, _int]


_dp = ctypes.POINTER(ctypes.c_double)
lib.px_partition_cost_fit.restype = _int
lib.px_partition_cost_fit.argtypes = [_dp, _dp, _int, _dp]
lib.px_partition_cost_argmin.restype = _int
lib.px_partition_cost_argmin.argtypes = [_dp, _i64, _i64, _i64p, _dp]
lib.px_partition_search_next.restype = _int
lib.px_partition_search_next.argtypes = [_dp, _dp, _int, _i64, _i64, _i64p]


class PxError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("px status %d (%s): %s" % (status, lib.px_status_string(status).decode(), message))
        self.status = status


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PX_F32
    if t.dtype == torch.bfloat16:
        return PX_BF16
    raise TypeError("px takes float32 or bfloat16 values, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr_array(tensors: Sequence[torch.Tensor]):
    return (ctypes.c_void_p * max(1, len(tensors)))(*[t.data_ptr() for t in tensors])


class Context:
    """px_ctx: one per stream."""

    def __init__(self, device: int = 0):
        self._h = _vp()
        rc = lib.px_create(ctypes.byref(self._h), device)
        if rc != PX_OK:
            raise PxError(rc, "px_create failed")
        self.device = device

    def close(self) -> None:
        if self._h:
            lib.px_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int) -> None:
        if rc != PX_OK:
            raise PxError(rc, lib.px_last_error(self._h).decode())

    # ------------------------------------------------------------------ calls

    def px_device_status(self, stream=None) -> int:
        """Waits for the stream; returns PX_OK, PX_ERR_INDEX_OUT_OF_RANGE or PX_ERR_NOT_UNIQUE and clears the flag."""
        return lib.px_device_status(self._h, _stream(stream))

    def px_set_wait_limit(self, polls: int) -> None:
        """Polls before a workgroup gives up a bounded wait for another's count (0: at once)."""
        self._check(lib.px_set_wait_limit(self._h, polls))

    @staticmethod
    def px_coalesce_scratch_bytes(total_rows: int, dim: int) -> int:
        return lib.px_coalesce_scratch_bytes(total_rows, dim)

    @staticmethod
    def px_partition_scratch_bytes(cap: int) -> int:
        return lib.px_partition_scratch_bytes(cap)

    def px_sparse_coalesce(self, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], dim: int,
                           vocab: int, scale: float, out_ids: torch.Tensor, out_rows: torch.Tensor,
                           out_num_unique: torch.Tensor, out_run_len: Optional[torch.Tensor],
                           scratch: torch.Tensor, stream=None) -> None:
        n, code, counts = self._coalesce_inputs(idx, val, dim)
        self._check(lib.px_sparse_coalesce(
            self._h, n, _ptr_array(idx), _ptr_array(val), counts, dim, code, vocab, scale,
            _ptr(out_ids), _ptr(out_rows), _ptr(out_num_unique), _ptr(out_run_len), _ptr(scratch),
            scratch.numel() * scratch.element_size(), _stream(stream)))

    @staticmethod
    def _coalesce_inputs(idx, val, dim):
        """Worker count, value dtype code and the host array of per-worker row counts."""
        n = len(idx)
        assert len(val) == n and n >= 1
        code = _dtype_code(val[0])
        counts = (ctypes.c_int64 * n)(*[int(i.numel()) for i in idx])
        for i, v in zip(idx, val):
            assert i.dtype == torch.int64 and i.is_contiguous() and v.is_contiguous()
            assert _dtype_code(v) == code and v.numel() == i.numel() * dim
        return n, code, counts

    def px_sparse_coalesce_apply_sgd(self, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor],
                                     vocab: int, scale: float, table: torch.Tensor, lr: float,
                                     out_ids: torch.Tensor, out_num_unique: torch.Tensor,
                                     out_run_len: Optional[torch.Tensor], scratch: torch.Tensor,
                                     stream=None) -> None:
        assert table.dtype == torch.float32 and table.is_contiguous() and table.shape[0] == vocab
        dim = table.shape[1]
        n, code, counts = self._coalesce_inputs(idx, val, dim)
        self._check(lib.px_sparse_coalesce_apply_sgd(
            self._h, n, _ptr_array(idx), _ptr_array(val), counts, dim, code, vocab, scale, _ptr(table), lr,
            _ptr(out_ids), _ptr(out_num_unique), _ptr(out_run_len), _ptr(scratch),
            scratch.numel() * scratch.element_size(), _stream(stream)))

    def px_sparse_coalesce_apply_adagrad(self, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor],
                                         vocab: int, scale: float, table: torch.Tensor,
                                         accum: torch.Tensor, lr: float, eps: float,
                                         out_ids: torch.Tensor, out_num_unique: torch.Tensor,
                                         out_run_len: Optional[torch.Tensor], scratch: torch.Tensor,
                                         stream=None) -> None:
        assert table.dtype == torch.float32 and table.is_contiguous() and table.shape[0] == vocab
        assert accum.dtype == torch.float32 and accum.is_contiguous() and accum.shape == table.shape
        dim = table.shape[1]
        n, code, counts = self._coalesce_inputs(idx, val, dim)
        self._check(lib.px_sparse_coalesce_apply_adagrad(
            self._h, n, _ptr_array(idx), _ptr_array(val), counts, dim, code, vocab, scale, _ptr(table),
            _ptr(accum), lr, eps, _ptr(out_ids), _ptr(out_num_unique), _ptr(out_run_len), _ptr(scratch),
            scratch.numel() * scratch.element_size(), _stream(stream)))

    def px_partition_rows(self, ids: torch.Tensor, num_ids: torch.Tensor, cap: int, num_shards: int,
                          hash: int, out_shard: Optional[torch.Tensor], out_perm: torch.Tensor,
                          out_offsets: torch.Tensor, scratch: torch.Tensor, stream=None) -> None:
        self._check(lib.px_partition_rows(
            self._h, _ptr(ids), _ptr(num_ids), cap, num_shards, hash, _ptr(out_shard), _ptr(out_perm),
            _ptr(out_offsets), _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))

    def px_partition_rows_noalloc(self, ids: torch.Tensor, num_ids: torch.Tensor, cap: int, num_shards: int,
                                  hash: int, out_shard: Optional[torch.Tensor], out_perm: torch.Tensor,
                                  out_offsets: torch.Tensor, stream=None) -> None:
        """px_partition_rows on the library's built-in scratch: allocates nothing, cap limited."""
        self._check(lib.px_partition_rows_noalloc(
            self._h, _ptr(ids), _ptr(num_ids), cap, num_shards, hash, _ptr(out_shard), _ptr(out_perm),
            _ptr(out_offsets), _stream(stream)))

    def px_sparse_apply_sgd(self, table: torch.Tensor, ids: torch.Tensor, rows: torch.Tensor,
                            num_ids: torch.Tensor, cap: int, perm: Optional[torch.Tensor],
                            range_: Optional[torch.Tensor], lr: float, stream=None) -> None:
        vocab, dim = table.shape
        assert table.dtype == torch.float32 and table.is_contiguous()
        self._check(lib.px_sparse_apply_sgd(
            self._h, _ptr(table), vocab, dim, _ptr(ids), _ptr(rows), _ptr(num_ids), cap, _ptr(perm),
            _ptr(range_), lr, _stream(stream)))

    def px_sparse_apply_adagrad(self, table: torch.Tensor, accum: torch.Tensor, ids: torch.Tensor,
                                rows: torch.Tensor, num_ids: torch.Tensor, cap: int,
                                perm: Optional[torch.Tensor], range_: Optional[torch.Tensor], lr: float,
                                eps: float = 0.0, stream=None) -> None:
        vocab, dim = table.shape
        assert table.dtype == torch.float32 and table.is_contiguous()
        assert accum.dtype == torch.float32 and accum.is_contiguous() and accum.shape == table.shape
        self._check(lib.px_sparse_apply_adagrad(
            self._h, _ptr(table), _ptr(accum), vocab, dim, _ptr(ids), _ptr(rows), _ptr(num_ids), cap,
            _ptr(perm), _ptr(range_), lr, eps, _stream(stream)))

    def px_sparse_lookup(self, table: torch.Tensor, ids: torch.Tensor, num_ids: Optional[torch.Tensor],
                         cap: int, perm: Optional[torch.Tensor], range_: Optional[torch.Tensor],
                         out_rows: torch.Tensor, stream=None) -> None:
        vocab, dim = table.shape
        assert table.dtype == torch.float32 and table.is_contiguous()
        assert out_rows.dtype == torch.float32 and out_rows.is_contiguous() and out_rows.numel() >= cap * dim
        assert ids.dtype == torch.int64 and ids.is_contiguous() and ids.numel() >= cap
        self._check(lib.px_sparse_lookup(self._h, _ptr(table), vocab, dim, _ptr(ids), _ptr(num_ids), cap,
                                         _ptr(perm), _ptr(range_), _ptr(out_rows), _stream(stream)))

    def px_dense_average(self, bufs: Sequence[torch.Tensor], count: int, out: torch.Tensor, scale: float,
                         stream=None) -> None:
        n = len(bufs)
        assert n >= 1
        code = _dtype_code(bufs[0])
        for b in bufs:
            assert _dtype_code(b) == code and b.is_contiguous() and b.numel() >= count
        assert out.is_contiguous() and out.numel() >= count
        self._check(lib.px_dense_average(self._h, n, _ptr_array(bufs), count, code, _ptr(out),
                                         _dtype_code(out), scale, _stream(stream)))


def px_dense_average_launches(n_buffers: int, count: int, in_bf16: bool, out_bf16: bool = False) -> int:
    """Kernel launches of the 128-bit path one px_dense_average call makes (host arithmetic)."""
    return int(lib.px_dense_average_launches(n_buffers, count, PX_BF16 if in_bf16 else PX_F32,
                                             PX_BF16 if out_bf16 else PX_F32))


def _doubles(values):
    return (ctypes.c_double * max(1, len(values)))(*[float(v) for v in values])


def px_partition_cost_fit(p: Sequence[float], t: Sequence[float]):
    """theta of Eq. 1 fitted to the samples (host arithmetic)."""
    theta = (ctypes.c_double * 3)()
    rc = lib.px_partition_cost_fit(_doubles(p), _doubles(t), len(p), theta)
    if rc != PX_OK:
        raise PxError(rc, "cost model fit needs three distinct positive partition counts")
    return [theta[0], theta[1], theta[2]]


def px_partition_cost_argmin(theta: Sequence[float], p_lo: int, p_hi: int):
    best, when = ctypes.c_int64(), ctypes.c_double()
    rc = lib.px_partition_cost_argmin(_doubles(theta), p_lo, p_hi, ctypes.byref(best), ctypes.byref(when))
    if rc != PX_OK:
        raise PxError(rc, "bad range")
    return best.value, when.value


def px_partition_search_next(p: Sequence[float], t: Sequence[float], p_start: int, p_max: int) -> int:
    nxt = ctypes.c_int64()
    rc = lib.px_partition_search_next(_doubles(p), _doubles(t), len(p), p_start, p_max, ctypes.byref(nxt))
    if rc != PX_OK:
        raise PxError(rc, "bad search arguments")
    return nxt.value


def alloc_scratch(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least nbytes (torch allocations are 256-byte aligned or better)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
