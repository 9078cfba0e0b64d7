"""Pins for the CPU oracle: checks that do not go through the oracle's own code.

Each ``pin_*`` function takes the loaded oracle library and raises
AssertionError when the oracle disagrees with something fixed from outside it:
brute-force densification, invariants, bit-exact special cases, closed forms,
Python big-integer arithmetic, numpy / PyTorch CPU library routines.
``tests/test_oracle_pins.py`` runs them against the real oracle;
``tests/test_oracle_mutants.py`` runs them against deliberately broken copies
of the oracle source and requires every planted mistake to be caught.
"""

from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_1808_02621_amd import inputs

RNG = np.random.default_rng


def _ulp_close(a, b, ulps=1):
    a = np.asarray(a, dtype=np.float32)
    b = np.asarray(b, dtype=np.float32)
    tol = ulps * np.spacing(np.maximum(np.abs(a), np.abs(b)).astype(np.float32))
    assert np.all(np.abs(a.astype(np.float64) - b.astype(np.float64)) <= tol), \
        "max diff %g" % np.max(np.abs(a.astype(np.float64) - b.astype(np.float64)))


def _densify_loops(idx, val, vocab, dim):
    """Brute force: every worker's gradient written out as a full [V, D] table, tables summed."""
    total = np.zeros((vocab, dim), dtype=np.float64)
    touched = np.zeros(vocab, dtype=bool)
    for i_w, v_w in zip(idx, val):
        dense_w = np.zeros((vocab, dim), dtype=np.float64)
        for r in range(len(i_w)):
            for d in range(dim):
                dense_w[i_w[r], d] += float(v_w[r, d])
            touched[i_w[r]] = True
        total += dense_w
    return total, touched


def _random_case(seed, vocab, dim, n_workers, max_rows, integer=False):
    rng = RNG(seed)
    idx, val = [], []
    for _ in range(n_workers):
        n = int(rng.integers(0, max_rows + 1))
        idx.append(rng.integers(0, vocab, size=n, dtype=np.int64))
        if integer:
            val.append(inputs.small_integer_values(rng, (n, dim)))
        else:
            val.append(rng.standard_normal((n, dim), dtype=np.float32))
    return idx, val


# ------------------------------------------------------------------- coalesce

def pin_coalesce_bruteforce_fuzz(lib):
    for seed in range(12):
        vocab = 1 + seed * 5
        dim = 1 + seed % 4
        idx, val = _random_case(seed, vocab, dim, n_workers=1 + seed % 5, max_rows=40)
        ids, rows, run_len = oracle.sparse_coalesce(idx, val, dim, vocab, lib=lib)
        total, touched = _densify_loops(idx, val, vocab, dim)
        assert np.array_equal(ids, np.nonzero(touched)[0])
        assert np.array_equal(rows, total[touched].astype(np.float32))
        counts = np.bincount(np.concatenate(idx), minlength=vocab) if ids.size else np.zeros(vocab)
        assert np.array_equal(run_len, counts[touched])


def pin_coalesce_bruteforce_tiny_config(lib):
    w = inputs.TINY
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    ids, rows, run_len = oracle.sparse_coalesce(idx, val, w.dim, w.vocab, lib=lib)
    total = np.zeros((w.vocab, w.dim), dtype=np.float64)
    for i_w, v_w in zip(idx, val):
        np.add.at(total, i_w, v_w.astype(np.float64))
    allids = np.concatenate(idx)
    touched = np.zeros(w.vocab, dtype=bool)
    touched[allids] = True
    assert ids.size == len(set(allids.tolist()))
    assert np.array_equal(ids, np.nonzero(touched)[0])
    assert np.all(total[~touched] == 0.0)
    _ulp_close(rows, total[touched].astype(np.float32))   # np.add.at's order may differ
    assert int(run_len.sum()) == allids.size


def pin_coalesce_invariants(lib):
    w = inputs.shrink(inputs.SMALL_LM, vocab=5000, n_per_worker=300, dim=24)
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    ids, rows, run_len = oracle.sparse_coalesce(idx, val, w.dim, w.vocab, lib=lib)
    allids = np.concatenate(idx)
    assert ids.size == len(set(allids.tolist()))
    assert np.all(np.diff(ids) > 0)
    assert int(run_len.sum()) == allids.size and np.all(run_len >= 1)
    col_in = np.concatenate(val).astype(np.float64).sum(axis=0)
    col_out = rows.astype(np.float64).sum(axis=0)
    assert np.allclose(col_in, col_out, rtol=0, atol=1e-3)
    # the hottest id of a Zipf draw is rank 1 -> id 0, and it is the longest run
    assert ids[0] == 0 and run_len[0] == run_len.max()


def pin_coalesce_all_distinct(lib):
    rng = RNG(5)
    vocab, dim = 997, 7
    perm = rng.permutation(vocab)[:600].astype(np.int64)
    vals = rng.standard_normal((600, dim), dtype=np.float32)
    idx = [perm[:200], perm[200:450], perm[450:]]
    val = [vals[:200], vals[200:450], vals[450:]]
    ids, rows, run_len = oracle.sparse_coalesce(idx, val, dim, vocab, lib=lib)
    order = np.argsort(perm)
    assert np.array_equal(ids, perm[order])
    assert np.array_equal(rows, vals[order])          # bit-exact: nothing is added
    assert np.all(run_len == 1)


def pin_coalesce_all_equal(lib):
    rng = RNG(6)
    dim = 5
    vals = [inputs.small_integer_values(rng, (n, dim)) for n in (17, 0, 40)]
    idx = [np.full(v.shape[0], 42, dtype=np.int64) for v in vals]
    ids, rows, run_len = oracle.sparse_coalesce(idx, vals, dim, 100, lib=lib)
    assert ids.tolist() == [42] and run_len.tolist() == [57]
    assert np.array_equal(rows[0], np.concatenate(vals).sum(axis=0))


def pin_coalesce_empty_and_single(lib):
    ids, rows, run_len = oracle.sparse_coalesce([], [], 4, 10, lib=lib)
    assert ids.size == 0 and rows.shape == (0, 4) and run_len.size == 0
    e = np.zeros(0, np.int64)
    ids, rows, _ = oracle.sparse_coalesce([e, e], [np.zeros((0, 4), np.float32)] * 2, 4, 10, lib=lib)
    assert ids.size == 0
    v = np.arange(12, dtype=np.float32).reshape(3, 4)
    ids, rows, run_len = oracle.sparse_coalesce([np.array([7, 2, 7])], [v], 4, 10, lib=lib)
    assert ids.tolist() == [2, 7] and run_len.tolist() == [1, 2]
    assert np.array_equal(rows, np.stack([v[1], v[0] + v[2]]))


def pin_coalesce_integer_exact(lib):
    # integer-valued rows: every partial sum is exact in float32, so any order gives the same bits
    rng = RNG(7)
    vocab, dim = 50, 6
    idx = [inputs.draw_ids(rng, vocab, 1.3, 4000) for _ in range(3)]
    val = [inputs.small_integer_values(rng, (4000, dim)) for _ in range(3)]
    ids, rows, _ = oracle.sparse_coalesce(idx, val, dim, vocab, lib=lib)
    total = np.zeros((vocab, dim), dtype=np.int64)
    for i_w, v_w in zip(idx, val):
        np.add.at(total, i_w, v_w.astype(np.int64))
    assert np.array_equal(rows, total[ids].astype(np.float32))
    # worker order does not matter
    ids2, rows2, _ = oracle.sparse_coalesce(idx[::-1], val[::-1], dim, vocab, lib=lib)
    assert np.array_equal(ids, ids2) and np.array_equal(rows, rows2)


def pin_coalesce_torch_library(lib):
    w = inputs.shrink(inputs.LARGE_LM, vocab=3000, n_workers=6, n_per_worker=500, dim=16)
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    ids, rows, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab, lib=lib)
    i = torch.from_numpy(np.concatenate(idx)).unsqueeze(0)
    v = torch.from_numpy(np.concatenate(val)).double()
    c = torch.sparse_coo_tensor(i, v, (w.vocab, w.dim)).coalesce()
    assert np.array_equal(ids, c.indices()[0].numpy())
    _ulp_close(rows, c.values().float().numpy())
    uniq, inv = torch.unique(i[0], sorted=True, return_inverse=True)
    acc = torch.zeros(uniq.numel(), w.dim, dtype=torch.float64).index_add_(0, inv, v)
    assert np.array_equal(ids, uniq.numpy())
    _ulp_close(rows, acc.float().numpy())


def pin_coalesce_average_is_over_workers(lib):
    rng = RNG(8)
    dim, n_workers = 3, 4
    idx = [np.array([1, 1, 5], dtype=np.int64) for _ in range(n_workers)]
    val = [inputs.small_integer_values(rng, (3, dim)) * np.float32(4.0) for _ in range(n_workers)]
    ids, s, _ = oracle.sparse_coalesce(idx, val, dim, 9, lib=lib)
    ids2, a, _ = oracle.sparse_coalesce(idx, val, dim, 9, average=True, lib=lib)
    assert np.array_equal(ids, ids2)
    assert np.array_equal(a, s / np.float32(n_workers))    # id 1 occurs 8 times, still / 4


def pin_coalesce_idempotent_and_two_level(lib):
    w = inputs.shrink(inputs.LARGE_LM, vocab=2000, n_workers=48, n_per_worker=40, dim=8)
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    ids, rows, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab, lib=lib)
    ids2, rows2, rl2 = oracle.sparse_coalesce([ids], [rows], w.dim, w.vocab, lib=lib)
    assert np.array_equal(ids, ids2) and np.array_equal(rows, rows2) and np.all(rl2 == 1)
    # aggregation inside each machine first, then between machines (Sec. 4.3): 8 groups of 6
    gi, gv = [], []
    for g in range(8):
        a, b, _ = oracle.sparse_coalesce(idx[6 * g:6 * g + 6], val[6 * g:6 * g + 6], w.dim, w.vocab, lib=lib)
        gi.append(a)
        gv.append(b)
    ids3, rows3, _ = oracle.sparse_coalesce(gi, gv, w.dim, w.vocab, lib=lib)
    assert np.array_equal(ids, ids3)
    assert np.allclose(rows, rows3, rtol=1e-6, atol=1e-6)


def pin_coalesce_bf16_widening(lib):
    rng = RNG(9)
    dim = 8
    v32 = rng.standard_normal((300, dim), dtype=np.float32)
    bits = inputs.f32_to_bf16_bits(v32)
    # the patterns against torch's own bfloat16 rounding and widening
    tb = torch.from_numpy(v32).to(torch.bfloat16)
    assert np.array_equal(bits, tb.view(torch.int16).numpy().view(np.uint16))
    widened = tb.float().numpy()
    idx = [rng.integers(0, 20, size=300, dtype=np.int64)]
    a = oracle.sparse_coalesce(idx, [bits], dim, 20, lib=lib)
    b = oracle.sparse_coalesce(idx, [widened], dim, 20, lib=lib)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    d = oracle.dense_average([bits[:, 0].copy(), bits[:, 1].copy()], lib=lib)
    e = oracle.dense_average([widened[:, 0].copy(), widened[:, 1].copy()], lib=lib)
    assert np.array_equal(d, e)


def pin_coalesce_rejects_bad_ids(lib):
    v = np.ones((2, 2), np.float32)
    for bad in (-1, 10, 2 ** 40):
        try:
            oracle.sparse_coalesce([np.array([3, bad])], [v], 2, 10, lib=lib)
        except oracle.IdOutOfRange:
            continue
        raise AssertionError("id %d accepted" % bad)


# ------------------------------------------------------------------ partition

def _py_shard(i, p, hash):
    return ((i * 2654435761) % (1 << 64)) % p if hash == "mul" else i % p


def pin_partition_structure(lib):
    rng = RNG(10)
    ids = np.unique(rng.integers(0, 1 << 20, size=5000, dtype=np.int64))
    for hash in ("mod", "mul"):
        for p in (1, 2, 3, 7, 8, 16, 32, 100):
            shard, perm, off = oracle.partition_rows(ids, p, hash, lib=lib)
            assert shard.tolist() == [_py_shard(int(i), p, hash) for i in ids]
            assert off[0] == 0 and off[p] == ids.size and np.all(np.diff(off) >= 0)
            assert np.array_equal(np.sort(perm), np.arange(ids.size))       # each id exactly once
            for q in range(p):
                sl = perm[off[q]:off[q + 1]]
                assert np.all(shard[sl] == q)
                assert np.all(np.diff(sl) > 0)                              # stable: ascending id
            assert np.array_equal(np.diff(off), np.bincount(shard, minlength=p))


def pin_partition_hash_wraps_at_64_bits(lib):
    big = np.array([0, 1, 2 ** 31 - 1, 2 ** 31, 2 ** 32 + 5, 2 ** 40 + 123, 2 ** 62 + 99,
                    2 ** 63 - 1], dtype=np.int64)
    for p in (3, 5, 32, 1000):
        shard, _, _ = oracle.partition_rows(big, p, "mul", lib=lib)
        assert shard.tolist() == [_py_shard(int(i), p, "mul") for i in big]
    # 2654435761 = 1 mod 16: the multiplicative hash equals id mod P for P in {2,4,8,16}
    ids = np.arange(0, 4000, dtype=np.int64) * 7919
    for p in (2, 4, 8, 16):
        a, _, _ = oracle.partition_rows(ids, p, "mul", lib=lib)
        b, _, _ = oracle.partition_rows(ids, p, "mod", lib=lib)
        assert np.array_equal(a, b)
    a, _, _ = oracle.partition_rows(ids, 32, "mul", lib=lib)
    b, _, _ = oracle.partition_rows(ids, 32, "mod", lib=lib)
    assert not np.array_equal(a, b) and a[1] == (7919 * 17) % 32


def pin_partition_commutes_with_coalesce(lib):
    # the paper splits the incoming rows first and aggregates per partition (Sec. 3.2)
    w = inputs.shrink(inputs.SMALL_LM, vocab=800, n_per_worker=200, dim=4)
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    ids, rows, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab, lib=lib)
    p = 4
    _, perm, off = oracle.partition_rows(ids, p, "mul", lib=lib)
    for q in range(p):
        pi, pv = [], []
        for i_w, v_w in zip(idx, val):
            keep = np.array([_py_shard(int(i), p, "mul") == q for i in i_w], dtype=bool)
            pi.append(i_w[keep])
            pv.append(v_w[keep])
        qi, qr, _ = oracle.sparse_coalesce(pi, pv, w.dim, w.vocab, lib=lib)
        sl = perm[off[q]:off[q + 1]]
        assert np.array_equal(qi, ids[sl]) and np.array_equal(qr, rows[sl])


# ------------------------------------------------------------------------ SGD

def pin_sgd_dense_equivalent(lib):
    rng = RNG(11)
    vocab, dim, lr = 300, 6, 0.05
    idx, val = _random_case(11, vocab, dim, n_workers=3, max_rows=200)
    ids, rows, _ = oracle.sparse_coalesce(idx, val, dim, vocab, lib=lib)
    table0 = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    table = table0.copy()
    oracle.sparse_apply_sgd(table, ids, rows, lr, lib=lib)
    dense = np.zeros((vocab, dim), dtype=np.float64)
    dense[ids] = rows
    ref = (table0.astype(np.float64) - lr * dense).astype(np.float32)
    assert np.array_equal(table, ref)
    untouched = np.ones(vocab, dtype=bool)
    untouched[ids] = False
    assert np.array_equal(table[untouched], table0[untouched]) and untouched.any()
    # linearity: applying the un-aggregated duplicates one by one lands within rounding
    seq = table0.astype(np.float64)
    for i_w, v_w in zip(idx, val):
        for r in range(len(i_w)):
            seq[i_w[r]] -= lr * v_w[r].astype(np.float64)
    assert np.allclose(table, seq, rtol=1e-6, atol=1e-6)
    # lr = 0 changes nothing; shard order (perm) does not change the result
    t2 = table0.copy()
    oracle.sparse_apply_sgd(t2, ids, rows, 0.0, lib=lib)
    assert np.array_equal(t2, table0)
    _, perm, _ = oracle.partition_rows(ids, 5, "mul", lib=lib)
    t3 = table0.copy()
    oracle.sparse_apply_sgd(t3, ids, rows, lr, perm=perm, lib=lib)
    assert np.array_equal(t3, table)
    # a perm that is not the identity must move whole (id, row) pairs together
    t4 = table0.copy()
    oracle.sparse_apply_sgd(t4, ids, rows, lr, perm=perm[::-1].copy(), lib=lib)
    assert np.array_equal(t4, table)


def pin_sgd_torch_library(lib):
    rng = RNG(12)
    vocab, dim, lr = 64, 5, 0.1
    ids = np.sort(rng.permutation(vocab)[:20]).astype(np.int64)
    rows = rng.standard_normal((20, dim), dtype=np.float32)
    table0 = rng.standard_normal((vocab, dim), dtype=np.float32)
    table = table0.copy()
    oracle.sparse_apply_sgd(table, ids, rows, lr, lib=lib)
    p = torch.nn.Parameter(torch.from_numpy(table0.copy()))
    opt = torch.optim.SGD([p], lr=lr)
    p.grad = torch.sparse_coo_tensor(torch.from_numpy(ids).unsqueeze(0), torch.from_numpy(rows),
                                     (vocab, dim))
    opt.step()
    assert np.allclose(table, p.detach().numpy(), rtol=1e-6, atol=1e-7)
    assert not np.array_equal(table, table0)


def pin_apply_rejects_bad_input(lib):
    table = np.zeros((10, 2), np.float32)
    rows = np.ones((2, 2), np.float32)
    for fn in (lambda i: oracle.sparse_apply_sgd(table, i, rows, 0.1, lib=lib),
               lambda i: oracle.sparse_apply_adagrad(table, table.copy() + 1, i, rows, 0.1, lib=lib)):
        for ids, exc in ((np.array([3, 3]), oracle.RepeatedId), (np.array([3, 10]), oracle.IdOutOfRange),
                         (np.array([-1, 3]), oracle.IdOutOfRange)):
            try:
                fn(ids.astype(np.int64))
            except exc:
                continue
            raise AssertionError("accepted %s" % ids)
    assert np.all(table == 0)


# -------------------------------------------------------------------- Adagrad

def pin_adagrad_closed_form(lib):
    rng = RNG(13)
    vocab, dim, lr, a0 = 40, 4, 0.2, 0.1
    ids = np.array([3, 7, 8, 30], dtype=np.int64)
    g = rng.standard_normal((4, dim), dtype=np.float32)
    g[2] = 0.0
    w0 = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    table, accum = w0.copy(), np.full((vocab, dim), a0, dtype=np.float32)
    oracle.sparse_apply_adagrad(table, accum, ids, g, lr, lib=lib)
    g64, a064 = g.astype(np.float64), np.float64(np.float32(a0))
    assert np.allclose(accum[ids], a064 + g64 ** 2, rtol=1e-7, atol=0)
    assert np.allclose(table[ids], w0[ids] - lr * g64 / np.sqrt(a064 + g64 ** 2), rtol=1e-6, atol=1e-8)
    assert np.all(np.abs(table[ids].astype(np.float64) - w0[ids]) < lr)
    assert np.array_equal(table[8], w0[8]) and np.all(accum[8] == np.float32(a0))    # g = 0
    rest = np.ones(vocab, dtype=bool)
    rest[ids] = False
    assert np.array_equal(table[rest], w0[rest]) and np.all(accum[rest] == np.float32(a0))
    # a second step with the same gradient: A = a0 + 2 g^2
    t1 = table.copy()
    oracle.sparse_apply_adagrad(table, accum, ids, g, lr, lib=lib)
    assert np.allclose(accum[ids], a064 + 2 * g64 ** 2, rtol=1e-6, atol=0)
    assert np.allclose(table[ids], t1[ids] - lr * g64 / np.sqrt(a064 + 2 * g64 ** 2), rtol=1e-6, atol=1e-8)
    # eps is added outside the square root
    t5, a5 = w0.copy(), np.full((vocab, dim), a0, dtype=np.float32)
    oracle.sparse_apply_adagrad(t5, a5, ids, g, lr, eps=0.5, lib=lib)
    assert np.allclose(t5[ids], w0[ids] - lr * g64 / (np.sqrt(a064 + g64 ** 2) + 0.5), rtol=1e-6, atol=1e-8)


def pin_adagrad_aggregates_before_update(lib):
    # one update from the aggregated row differs from one update per duplicate (it is not linear)
    dim, lr, a0 = 2, 0.2, 0.1
    idx = [np.array([5, 5], dtype=np.int64)]
    val = [np.array([[1.0, 2.0], [1.0, -1.0]], dtype=np.float32)]
    ids, rows, _ = oracle.sparse_coalesce(idx, val, dim, 10, lib=lib)
    table, accum = np.zeros((10, dim), np.float32), np.full((10, dim), a0, np.float32)
    oracle.sparse_apply_adagrad(table, accum, ids, rows, lr, lib=lib)
    g = np.array([2.0, 1.0])
    assert np.allclose(accum[5], a0 + g ** 2, rtol=1e-6)
    assert np.allclose(table[5], -lr * g / np.sqrt(a0 + g ** 2), rtol=1e-6)
    per_dup = np.zeros(dim)
    acc = np.full(dim, a0)
    for r in val[0].astype(np.float64):
        acc += r ** 2
        per_dup -= lr * r / np.sqrt(acc)
    assert not np.allclose(table[5], per_dup, rtol=1e-3)


def pin_adagrad_torch_library(lib):
    rng = RNG(14)
    vocab, dim, lr = 50, 6, 0.2
    table0 = rng.standard_normal((vocab, dim), dtype=np.float32)
    table, accum = table0.copy(), np.full((vocab, dim), 0.1, dtype=np.float32)
    p = torch.nn.Parameter(torch.from_numpy(table0.copy()))
    opt = torch.optim.Adagrad([p], lr=lr, initial_accumulator_value=0.1, eps=1e-10)
    for step in range(3):
        ids = np.sort(rng.permutation(vocab)[:15]).astype(np.int64)
        rows = rng.standard_normal((15, dim), dtype=np.float32)
        _, perm, _ = oracle.partition_rows(ids, 4, "mul", lib=lib)
        oracle.sparse_apply_adagrad(table, accum, ids, rows, lr, perm=perm, lib=lib)
        p.grad = torch.sparse_coo_tensor(torch.from_numpy(ids).unsqueeze(0),
                                         torch.from_numpy(rows), (vocab, dim))
        opt.step()
    assert np.allclose(table, p.detach().numpy(), rtol=2e-6, atol=1e-7)
    assert np.allclose(accum, opt.state[p]["sum"].numpy(), rtol=1e-6, atol=0)


# --------------------------------------------------------------------- lookup

def pin_lookup_is_an_indexed_copy(lib):
    rng = RNG(16)
    vocab, dim, n = 90, 5, 400
    table = rng.standard_normal((vocab, dim), dtype=np.float32)
    ids = inputs.draw_ids(rng, vocab, 1.1, n)                      # repeats on purpose
    out = oracle.sparse_lookup(table, ids, lib=lib)
    assert np.array_equal(out, table[ids])                          # numpy fancy indexing
    assert np.array_equal(out, np.take(table, ids, axis=0))
    # shard by shard (the partitioned lookup), stitched by position: same tensor
    p = 6
    _, perm, off = oracle.partition_rows(ids, p, "mul", lib=lib)
    stitched = np.full((n, dim), np.nan, dtype=np.float32)
    for q in range(p):
        before = stitched.copy()
        oracle.sparse_lookup(table, ids, perm=perm, first=int(off[q]), last=int(off[q + 1]), out=stitched, lib=lib)
        mine = perm[off[q]:off[q + 1]]
        others = np.setdiff1d(np.arange(n), mine)
        assert np.array_equal(stitched[others], before[others], equal_nan=True)   # a shard writes only its rows
        assert np.array_equal(stitched[mine], table[ids[mine]])
    assert np.array_equal(stitched, out)
    # the lookup inverts the update's addressing: rows pulled after an SGD step are the updated rows
    uids, rows, _ = oracle.sparse_coalesce([ids], [rng.standard_normal((n, dim), dtype=np.float32)], dim, vocab, lib=lib)
    t2 = table.copy()
    oracle.sparse_apply_sgd(t2, uids, rows, 0.5, lib=lib)
    assert np.array_equal(oracle.sparse_lookup(t2, uids, lib=lib), t2[uids])
    try:
        oracle.sparse_lookup(table, np.array([1, vocab]), lib=lib)
    except oracle.IdOutOfRange:
        pass
    else:
        raise AssertionError("bad id accepted")


# ---------------------------------------------------------------------- dense

def pin_dense_special_cases(lib):
    rng = RNG(15)
    x = rng.standard_normal(1000, dtype=np.float32)
    assert np.array_equal(oracle.dense_average([x], lib=lib), x)                   # N = 1
    assert np.array_equal(oracle.dense_average([x] * 4, lib=lib), x)               # all equal
    assert np.array_equal(oracle.dense_average([x] * 4, average=False, lib=lib), x * np.float32(4))
    ints = [inputs.small_integer_values(rng, (1000,), -100, 100) for _ in range(8)]
    exact = np.sum(np.stack(ints).astype(np.int64), axis=0)
    assert np.array_equal(oracle.dense_average(ints, average=False, lib=lib), exact.astype(np.float32))
    assert np.array_equal(oracle.dense_average(ints, lib=lib), (exact / 8.0).astype(np.float32))


def pin_dense_numpy_mean(lib):
    w = inputs.shrink(inputs.LARGE_LM, n_workers=7, dense_count=4099)
    bufs = inputs.dense_buffers(w)
    ref = np.mean(np.stack(bufs), axis=0, dtype=np.float64)
    _ulp_close(oracle.dense_average(bufs, lib=lib), ref.astype(np.float32))
    ref = np.sum(np.stack(bufs), axis=0, dtype=np.float64)
    _ulp_close(oracle.dense_average(bufs, average=False, lib=lib), ref.astype(np.float32))
    w = inputs.shrink(inputs.NMT, n_workers=5, dense_count=1031)
    bits = inputs.dense_buffers(w)
    wide = np.stack([torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).double().numpy() for b in bits])
    _ulp_close(oracle.dense_average(bits, lib=lib), wide.mean(axis=0).astype(np.float32))


# structural pins first: a broken perm or offset must be caught before anything indexes with it
ALL_PINS = sorted((v for k, v in globals().items() if k.startswith("pin_") and callable(v)),
                  key=lambda f: (not f.__name__.startswith("pin_partition"), f.__name__))
