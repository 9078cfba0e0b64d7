"""px_partition_rows_noalloc (the entry point that allocates nothing: its workspace is an array
built into the library) against px_partition_rows, through the C ABI, on an MI355X.

Two calls in a row on the same GPU, the second with a smaller input, must each give exactly
what the workspace-taking entry point gives (shard numbers, perm, offsets: bit-exact), which
the other GPU tests check against the oracle; the oracle is consulted here as well.
"""

import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def _ids(rng, n, vocab):
    return np.unique(rng.integers(0, vocab, size=n, dtype=np.int64))          # ascending, distinct, at most n


def _both(ctx, px, ids, cap, n_shards, hash_code, hash_name):
    n = ids.size
    d_ids = torch.full((cap,), -7, dtype=torch.int64, device="cuda")
    d_ids[:n] = torch.from_numpy(ids).cuda()
    num = torch.tensor([n], dtype=torch.int64, device="cuda")
    outs = []
    for variant in ("workspace", "noalloc"):
        shard = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        perm = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        offsets = torch.full((n_shards + 1,), -1, dtype=torch.int64, device="cuda")
        if variant == "workspace":
            work = px.alloc_scratch(px.Context.px_partition_scratch_bytes(cap))
            ctx.px_partition_rows(d_ids, num, cap, n_shards, hash_code, shard, perm, offsets, work)
        else:
            ctx.px_partition_rows_noalloc(d_ids, num, cap, n_shards, hash_code, shard, perm, offsets)
        torch.cuda.synchronize()
        outs.append((shard[:n].cpu().numpy(), perm[:n].cpu().numpy(), offsets.cpu().numpy()))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    o_shard, o_perm, o_off = oracle.partition_rows(ids, n_shards, hash_name)
    assert np.array_equal(outs[1][0], o_shard) and np.array_equal(outs[1][1], o_perm)
    assert np.array_equal(outs[1][2], o_off)


def test_noalloc_partition_matches_the_workspace_entry_point_twice_in_a_row():
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_1808_02621_amd import px
    ctx = px.Context(0)
    rng = np.random.default_rng(1808)
    # a large input over many sort blocks (prefix kernel path), then a small one (single launch pair),
    # then the large shape again with another shard count: the array keeps the earlier calls' contents
    _both(ctx, px, _ids(rng, 300_000, 4_000_000), 400_000, 16, px.PX_HASH_MUL, "mul")
    _both(ctx, px, _ids(rng, 5_000, 800_000), 6_000, 8, px.PX_HASH_MOD, "mod")
    _both(ctx, px, _ids(rng, 70_000, 1 << 32), 70_001, 100, px.PX_HASH_MUL, "mul")
    _both(ctx, px, np.zeros(0, dtype=np.int64), 3, 4, px.PX_HASH_MOD, "mod")
    assert ctx.px_device_status() == px.PX_OK
    # a second context on the same GPU uses the same array
    other = px.Context(0)
    _both(other, px, _ids(rng, 9_000, 50_000), 9_000, 7, px.PX_HASH_MUL, "mul")
    other.close()
    # a cap beyond what the built-in scratch serves is refused on the host, outputs untouched
    cap = px.PX_PARTITION_NOALLOC_MAX_IDS + 1
    perm = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ids = torch.zeros(8, dtype=torch.int64, device="cuda")
    num = torch.tensor([8], dtype=torch.int64, device="cuda")
    with pytest.raises(px.PxError) as err:
        ctx.px_partition_rows_noalloc(ids, num, cap, 2, px.PX_HASH_MOD, None, perm, offsets)
    assert err.value.status == px.PX_ERR_INVALID_ARG and "px_partition_rows" in str(err.value)
    torch.cuda.synchronize()
    assert bool((perm == -1).all()) and bool((offsets == -1).all())
    ctx.close()
