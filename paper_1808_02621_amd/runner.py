"""Device-buffer plumbing around the px entry points: allocate, upload, call in order.

Used by the tests, the smoke check and the benchmark so that all three drive the
library the same way.  No arithmetic of the method happens here.
"""

from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import px


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bfloat16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


@dataclasses.dataclass
class SparseBuffers:
    """Everything one sparse variable's coalesce -> partition -> apply chain touches on the device."""

    idx: List[torch.Tensor]
    val: List[torch.Tensor]
    dim: int
    vocab: int
    total_rows: int
    out_ids: torch.Tensor
    out_rows: torch.Tensor
    out_num: torch.Tensor
    out_run_len: torch.Tensor
    scratch: torch.Tensor
    shard: torch.Tensor
    perm: torch.Tensor
    offsets: torch.Tensor
    part_scratch: torch.Tensor
    n_shards: int
    hash: int


def sparse_buffers(idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], dim: int, vocab: int,
                   n_shards: int, hash: int, device="cuda") -> SparseBuffers:
    m = int(sum(int(i.numel()) for i in idx))
    cap = max(m, 1)
    return SparseBuffers(
        idx=list(idx), val=list(val), dim=dim, vocab=vocab, total_rows=m,
        out_ids=torch.empty(cap, dtype=torch.int64, device=device),
        out_rows=torch.empty((cap, dim), dtype=torch.float32, device=device),
        out_num=torch.zeros(1, dtype=torch.int64, device=device),
        out_run_len=torch.empty(cap, dtype=torch.int32, device=device),
        scratch=px.alloc_scratch(px.Context.px_coalesce_scratch_bytes(m, dim), device),
        shard=torch.empty(cap, dtype=torch.int32, device=device),
        perm=torch.empty(cap, dtype=torch.int32, device=device),
        offsets=torch.empty(n_shards + 1, dtype=torch.int64, device=device),
        part_scratch=px.alloc_scratch(px.Context.px_partition_scratch_bytes(m), device),
        n_shards=n_shards, hash=hash)


def coalesce(ctx: px.Context, b: SparseBuffers, scale: float = 1.0, stream=None) -> None:
    ctx.px_sparse_coalesce(b.idx, b.val, b.dim, b.vocab, scale, b.out_ids, b.out_rows, b.out_num,
                           b.out_run_len, b.scratch, stream)


def partition(ctx: px.Context, b: SparseBuffers, stream=None) -> None:
    # there are no more distinct ids than input rows, nor than rows in the table: the tighter bound
    # sizes the partition's launches
    cap = max(1, min(b.total_rows, b.vocab))
    ctx.px_partition_rows(b.out_ids, b.out_num, cap, b.n_shards, b.hash, b.shard, b.perm,
                          b.offsets, b.part_scratch, stream)


def apply(ctx: px.Context, b: SparseBuffers, table: torch.Tensor, accum: Optional[torch.Tensor],
          optimizer: str, lr: float, eps: float = 0.0, use_perm: bool = True,
          range_: Optional[torch.Tensor] = None, stream=None) -> None:
    perm = b.perm if use_perm else None
    # as for the partition: no more distinct ids than input rows, nor than rows in the table
    cap = max(1, min(b.total_rows, b.vocab))
    if optimizer == "sgd":
        ctx.px_sparse_apply_sgd(table, b.out_ids, b.out_rows, b.out_num, cap, perm, range_, lr, stream)
    elif optimizer == "adagrad":
        ctx.px_sparse_apply_adagrad(table, accum, b.out_ids, b.out_rows, b.out_num, cap, perm, range_, lr, eps,
                                    stream)
    else:
        raise ValueError(optimizer)


def sparse_step(ctx: px.Context, b: SparseBuffers, table: torch.Tensor, accum: Optional[torch.Tensor],
                optimizer: str, lr: float, scale: float = 1.0, stream=None) -> None:
    """coalesce -> partition -> apply (all shards), enqueued back to back."""
    coalesce(ctx, b, scale, stream)
    partition(ctx, b, stream)
    apply(ctx, b, table, accum, optimizer, lr, stream=stream)


def fused_step(ctx: px.Context, b: SparseBuffers, table: torch.Tensor, accum: Optional[torch.Tensor],
               optimizer: str, lr: float, scale: float = 1.0, eps: float = 0.0, stream=None) -> None:
    """Aggregate and update in one call (the aggregated rows are never stored), then partition the ids."""
    if optimizer == "sgd":
        ctx.px_sparse_coalesce_apply_sgd(b.idx, b.val, b.vocab, scale, table, lr, b.out_ids, b.out_num,
                                         b.out_run_len, b.scratch, stream)
    elif optimizer == "adagrad":
        ctx.px_sparse_coalesce_apply_adagrad(b.idx, b.val, b.vocab, scale, table, accum, lr, eps, b.out_ids,
                                             b.out_num, b.out_run_len, b.scratch, stream)
    else:
        raise ValueError(optimizer)
    partition(ctx, b, stream)


@dataclasses.dataclass
class TwoLevelBuffers:
    """Everything two-level aggregation touches, allocated once: one SparseBuffers per group of workers
    and one for the second level, sized for the case that no group combines anything."""

    firsts: List[SparseBuffers]
    second: SparseBuffers
    counts: torch.Tensor          # the groups' distinct-row counts, gathered for one read-back


def two_level_buffers(idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], dim: int, vocab: int,
                      group: int, device="cuda") -> TwoLevelBuffers:
    firsts = [sparse_buffers(idx[g0:g0 + group], val[g0:g0 + group], dim, vocab, 1, px.PX_HASH_MOD, device)
              for g0 in range(0, len(idx), group)]
    # the second level reads the first level's outputs in place; its own outputs and scratch are sized
    # for all of them being full
    second = sparse_buffers([b.out_ids for b in firsts], [b.out_rows for b in firsts], dim, vocab, 1,
                            px.PX_HASH_MOD, device)
    return TwoLevelBuffers(firsts, second, torch.zeros(len(firsts), dtype=torch.int64, device=device))


def two_level_first(ctx: px.Context, t: TwoLevelBuffers, stream=None) -> None:
    """Local aggregation: one coalesce per group of workers (Parallax Sec. 4.3), enqueued back to back."""
    for b in t.firsts:
        coalesce(ctx, b, 1.0, stream)


def two_level_read_counts(t: TwoLevelBuffers) -> List[int]:
    """The one synchronisation: the second call takes its row counts from the host."""
    torch.stack([b.out_num[0] for b in t.firsts], out=t.counts)
    return t.counts.cpu().tolist()


def two_level_second(ctx: px.Context, t: TwoLevelBuffers, counts: Sequence[int], stream=None) -> None:
    """Global aggregation of the groups' results (views of the first level's outputs, nothing is copied)."""
    t.second.idx = [b.out_ids[:n] for b, n in zip(t.firsts, counts)]
    t.second.val = [b.out_rows[:n] for b, n in zip(t.firsts, counts)]
    coalesce(ctx, t.second, 1.0, stream)


def two_level_coalesce(ctx: px.Context, idx: Sequence[torch.Tensor], val: Sequence[torch.Tensor], dim: int,
                       vocab: int, group: int, stream=None):
    """Aggregation in two levels (Parallax Sec. 4.3): first among the `group` workers of each machine,
    then across machines.  Returns the second level's SparseBuffers (ids, rows, count) and the list
    of first-level buffers.  The first-level counts are read back to the host in between (one
    synchronisation), because the second call takes its row counts from the host."""
    t = two_level_buffers(idx, val, dim, vocab, group)
    two_level_first(ctx, t, stream)
    two_level_second(ctx, t, two_level_read_counts(t), stream)
    return t.second, t.firsts
