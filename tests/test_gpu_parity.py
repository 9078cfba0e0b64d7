"""HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X).

Bars: ids, counts, run lengths, shard numbers, perm and offsets bit-exact;
float32 rows / tables / accumulators within |x - ref| <= 1e-6 + 1e-5 |ref|;
bf16-valued inputs within 1e-2 relative (they agree far more tightly, since both
sides widen exactly and accumulate wider than float32).
"""

import numpy as np
import pytest
import torch

import oracle
from paper_1808_02621_amd import inputs

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL = 1e-6, 1e-5


def close(x, ref, rel=REL_TOL, abs_=ABS_TOL):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bad = np.abs(x - ref) > abs_ + rel * np.abs(ref)
    assert not bad.any(), "%d of %d elements off, worst |diff| %g" % (
        int(bad.sum()), bad.size, float(np.max(np.abs(x - ref))))


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1808_02621_amd import px, runner
    ctx = px.Context(0)
    yield ctx, px, runner
    ctx.close()


def run_chain(gpu, idx, val, dim, vocab, n_shards, hash_name, optimizer, lr, table, accum=None,
              scale=1.0, check_rows_exact=False, rel=REL_TOL):
    """Runs coalesce -> partition -> apply on the GPU and on the oracle and compares everything."""
    ctx, px, runner = gpu
    hash_code = px.PX_HASH_MUL if hash_name == "mul" else px.PX_HASH_MOD
    d_idx = [runner.to_device(i) for i in idx]
    d_val = [runner.to_device(v).reshape(-1, dim) for v in val]
    b = runner.sparse_buffers(d_idx, d_val, dim, vocab, n_shards, hash_code)
    d_table = torch.from_numpy(table).cuda()
    d_accum = None if accum is None else torch.from_numpy(accum).cuda()
    runner.sparse_step(ctx, b, d_table, d_accum, optimizer, lr, scale)
    assert ctx.px_device_status() == px.PX_OK
    u = int(b.out_num.item())

    o_ids, o_rows, o_len = oracle.sparse_coalesce(idx, val, dim, vocab, average=False)
    if scale != 1.0:
        o_ids, o_rows, o_len = oracle.sparse_coalesce(idx, val, dim, vocab, average=True)
    assert u == o_ids.size
    assert np.array_equal(b.out_ids[:u].cpu().numpy(), o_ids)
    assert np.array_equal(b.out_run_len[:u].cpu().numpy(), o_len)
    g_rows = b.out_rows[:u].cpu().numpy()
    if check_rows_exact:
        assert np.array_equal(g_rows, o_rows)
    else:
        close(g_rows, o_rows, rel)
        # what the double accumulators actually deliver: both sides round the same real sum (formed in
        # double) once, so they are at most one unit in the last place apart; two when the sum is also
        # scaled, since the library multiplies by the float scale where the oracle divides by N
        ulp = np.spacing(np.maximum(np.abs(o_rows), np.float32(1e-30)))
        worst = float(np.max(np.abs(g_rows.astype(np.float64) - o_rows.astype(np.float64)) / ulp)) if o_rows.size else 0.0
        assert worst <= (1.0 if scale == 1.0 else 2.0), "aggregated rows up to %.1f ulp from the oracle" % worst

    o_shard, o_perm, o_off = oracle.partition_rows(o_ids, n_shards, hash_name)
    assert np.array_equal(b.shard[:u].cpu().numpy(), o_shard)
    assert np.array_equal(b.perm[:u].cpu().numpy(), o_perm)
    assert np.array_equal(b.offsets.cpu().numpy(), o_off)

    ref_table = table.copy()
    if optimizer == "sgd":
        oracle.sparse_apply_sgd(ref_table, o_ids, o_rows, lr, perm=o_perm)
    else:
        ref_accum = accum.copy()
        oracle.sparse_apply_adagrad(ref_table, ref_accum, o_ids, o_rows, lr, perm=o_perm)
        g_accum = d_accum.cpu().numpy()
        close(g_accum[o_ids], ref_accum[o_ids], rel)
    g_table = d_table.cpu().numpy()
    close(g_table[o_ids], ref_table[o_ids], rel)
    untouched = np.ones(vocab, dtype=bool)
    untouched[o_ids] = False
    assert np.array_equal(g_table[untouched], table[untouched])
    if accum is not None:
        assert np.array_equal(g_accum[untouched], accum[untouched])

    # the fused aggregate-and-apply entry points: same bits as the three separate calls
    f_table = torch.from_numpy(table).cuda()
    f_accum = None if accum is None else torch.from_numpy(accum).cuda()
    fb = runner.sparse_buffers(d_idx, d_val, dim, vocab, n_shards, hash_code)
    fb.out_rows.fill_(float("nan"))                      # never written by the fused path
    runner.fused_step(ctx, fb, f_table, f_accum, optimizer, lr, scale)
    assert ctx.px_device_status() == px.PX_OK
    assert int(fb.out_num.item()) == u
    assert torch.equal(fb.out_ids[:u], b.out_ids[:u]) and torch.equal(fb.out_run_len[:u], b.out_run_len[:u])
    assert torch.equal(fb.perm[:u], b.perm[:u]) and torch.equal(fb.offsets, b.offsets)
    assert torch.equal(f_table, d_table), "fused and separate paths differ in %d table elements" % int(
        (f_table != d_table).sum())
    if accum is not None:
        assert torch.equal(f_accum, d_accum)
    assert bool(torch.isnan(fb.out_rows).all())
    return b, u


def run_workload(gpu, w, table_index=0, permute=False, rel=REL_TOL):
    idx = inputs.sparse_ids(w, table_index, permute)
    val = inputs.sparse_values(w, table_index)
    table = inputs.table_init(w, table_index)
    accum = inputs.accum_init(w) if w.optimizer == "adagrad" else None
    return run_chain(gpu, idx, val, w.dim, w.vocab, w.n_shards, w.hash, w.optimizer, w.lr, table, accum,
                     rel=rel)


# ------------------------------------------------------------- the workloads

def test_tiny(gpu):
    run_workload(gpu, inputs.TINY)


def test_small_lm(gpu):
    run_workload(gpu, inputs.SMALL_LM)


def test_small_lm_scattered_hot_ids(gpu):
    run_workload(gpu, inputs.SMALL_LM, permute=True)


def test_large_lm_shrunk(gpu):
    run_workload(gpu, inputs.shrink(inputs.LARGE_LM, vocab=50_000, n_per_worker=300))


def test_nmt_shrunk_both_tables(gpu):
    w = inputs.shrink(inputs.NMT, n_workers=12, n_per_worker=1000)
    run_workload(gpu, w, 0, rel=1e-2)
    run_workload(gpu, w, 1, rel=1e-2)
    run_workload(gpu, w, 0)        # the agreement is in fact at the float32 bar


def test_stress_shrunk(gpu):
    run_workload(gpu, inputs.shrink(inputs.STRESS_UNIFORM, vocab=300_000, n_workers=16, n_per_worker=4000))
    run_workload(gpu, inputs.shrink(inputs.STRESS_ZIPF, vocab=300_000, n_workers=16, n_per_worker=4000))


def test_large_lm_full_size(gpu):
    run_workload(gpu, inputs.LARGE_LM)


def test_nmt_full_size(gpu):
    run_workload(gpu, inputs.NMT, 0)
    run_workload(gpu, inputs.NMT, 1)


def test_stress_full_size(gpu):
    run_workload(gpu, inputs.STRESS_UNIFORM)
    run_workload(gpu, inputs.STRESS_ZIPF)


def test_contexts_on_separate_streams_give_the_same_bits(gpu):
    """Two variables' chains and a dense mean enqueued side by side, one context and stream each."""
    ctx, px, runner = gpu
    w = inputs.shrink(inputs.NMT, n_workers=12, n_per_worker=3000, dense_count=1 << 20)
    hash_code = px.PX_HASH_MUL
    tables0 = [inputs.table_init(w, t) for t in range(2)]
    dev = []
    for t in range(2):
        d_idx = [runner.to_device(i) for i in inputs.sparse_ids(w, t)]
        d_val = [runner.to_device(v) for v in inputs.sparse_values(w, t)]
        dev.append((d_idx, d_val))
    d_dense = [runner.to_device(b) for b in inputs.dense_buffers(w)]

    def run(contexts, streams):
        outs = []
        bufs = [runner.sparse_buffers(i, v, w.dim, w.vocab, w.n_shards, hash_code) for i, v in dev]
        tabs = [torch.from_numpy(t0).cuda() for t0 in tables0]
        mean = torch.empty(w.dense_count, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        contexts[2].px_dense_average(d_dense, w.dense_count, mean, 1.0 / w.n_workers, streams[2])
        for t in range(2):
            runner.sparse_step(contexts[t], bufs[t], tabs[t], None, "sgd", w.lr, stream=streams[t])
        torch.cuda.synchronize()
        for c in set(contexts):
            assert c.px_device_status() == px.PX_OK
        for t in range(2):
            u = int(bufs[t].out_num.item())
            outs += [bufs[t].out_ids[:u].clone(), bufs[t].out_rows[:u].clone(), bufs[t].perm[:u].clone(), tabs[t]]
        return outs + [mean]

    serial = run([ctx, ctx, ctx], [None, None, None])
    side_ctx = [px.Context(0) for _ in range(3)]
    side_streams = [torch.cuda.Stream() for _ in range(3)]
    try:
        for _ in range(3):
            for a, b in zip(serial, run(side_ctx, side_streams)):
                assert torch.equal(a, b)
    finally:
        for c in side_ctx:
            c.close()
    # and the serial result is the oracle's
    o_ids, o_rows, _ = oracle.sparse_coalesce(inputs.sparse_ids(w, 0), inputs.sparse_values(w, 0), w.dim, w.vocab)
    assert np.array_equal(serial[0].cpu().numpy(), o_ids)
    close(serial[1].cpu().numpy(), o_rows)
    close(serial[8].cpu().numpy(), oracle.dense_average(inputs.dense_buffers(w), average=True))


# ------------------------------------------------------------------- shapes

@pytest.mark.parametrize("dim", [1, 3, 7, 8, 20, 64, 100, 132, 300, 1028, 2052])
@pytest.mark.parametrize("bf16", [False, True])
def test_row_widths(gpu, dim, bf16):
    rng = np.random.default_rng(dim * 2 + int(bf16))
    vocab, n_workers = 500, 5
    idx = [inputs.draw_ids(rng, vocab, 1.1, int(n)) for n in rng.integers(50, 400, size=n_workers)]
    val = [rng.standard_normal((i.size, dim), dtype=np.float32) for i in idx]
    if bf16:
        val = [inputs.f32_to_bf16_bits(v) for v in val]
    table = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    accum = np.full((vocab, dim), 0.1, dtype=np.float32)
    run_chain(gpu, idx, val, dim, vocab, 3, "mul", "adagrad", 0.1, table, accum)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(gpu, seed):
    """Random worker counts, ragged sizes, widths, vocabularies, skews, shard counts and optimizers."""
    rng = np.random.default_rng(1000 + seed)
    n_workers = int(rng.integers(1, 70))
    vocab = int(rng.choice([1, 2, 37, 500, 4096, 70_000, 1 << 20]))
    dim = int(rng.choice([1, 4, 5, 16, 36, 64, 96, 128, 200, 256, 384, 520, 1024]))
    budget = int(rng.choice([300, 5000, 60_000])) if dim <= 256 else int(rng.choice([300, 5000]))
    skew = rng.choice([None, 0.8, 1.0, 1.5, 2.5])
    sizes = rng.multinomial(budget, rng.dirichlet(np.ones(n_workers) * 0.5))
    idx = [inputs.draw_ids(rng, vocab, None if skew is None else float(skew), int(k)) for k in sizes]
    bf16 = bool(rng.integers(0, 2))
    val = [rng.standard_normal((int(k), dim), dtype=np.float32) for k in sizes]
    if bf16:
        val = [inputs.f32_to_bf16_bits(v) for v in val]
    table = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    optimizer = str(rng.choice(["sgd", "adagrad"]))
    accum = np.full((vocab, dim), 0.1, dtype=np.float32) if optimizer == "adagrad" else None
    n_shards = int(rng.choice([1, 2, 3, 8, 16, 31, 256]))
    scale = float(rng.choice([1.0, 1.0 / n_workers]))
    run_chain(gpu, idx, val, dim, vocab, n_shards, str(rng.choice(["mod", "mul"])), optimizer,
              float(rng.choice([0.01, 0.5])), table, accum, scale=scale)


RUN_LENGTHS = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 24, 31, 32, 33, 40, 63, 64, 65, 96, 127, 128, 129, 255, 257, 300]


@pytest.mark.parametrize("dim,bf16", [(128, False), (1024, True), (2048, False), (5, False), (40, True)])
def test_run_lengths_around_batch_and_window_borders(gpu, dim, bf16):
    """Runs whose lengths sit on and around the batch sizes (2, 4, 8) and the window sizes (32 ... 256),
    one run of several thousand rows in the middle, integer values: every row sum must be exact."""
    rng = np.random.default_rng(77 + dim)
    lengths = RUN_LENGTHS * 2 + [5000] + RUN_LENGTHS[::-1] * 2 + [1] * 700
    vocab = 4 * len(lengths)
    ids_of_runs = np.sort(rng.choice(vocab, size=len(lengths), replace=False))
    all_ids = np.repeat(ids_of_runs, lengths)
    rng.shuffle(all_ids)
    cuts = np.sort(rng.choice(all_ids.size, size=6, replace=False))
    idx = [a.astype(np.int64) for a in np.split(all_ids, cuts)]
    val = [inputs.small_integer_values(rng, (i.size, dim)) for i in idx]
    if bf16:
        val = [inputs.f32_to_bf16_bits(v) for v in val]
    table = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    accum = np.full((vocab, dim), 0.1, dtype=np.float32)
    b, u = run_chain(gpu, idx, val, dim, vocab, 5, "mul", "adagrad", 0.1, table, accum, check_rows_exact=True)
    assert u == len(lengths)


@pytest.mark.parametrize("rows", [1, 255, 1023, 1024, 1025, 2047, 2048, 2049, 4097, 32_768, 32_769, 1024 * 33, 65_536, 65_537, 2048 * 33, 2048 * 40 + 1, 262_144, 262_145])
def test_row_counts_around_the_one_launch_prefix_limit(gpu, rows):
    """Row counts on both sides of every switch of the sort's geometry: one tile (1,024 rows) and its
    multiples, 32 sort blocks (up to which the scatter sums the histogram rows itself; above, the
    prefix kernel runs), 256 blocks (wide digits up to there), and a ragged last tile."""
    rng = np.random.default_rng(rows)
    vocab, dim = 70_000, 4
    sizes = rng.multinomial(rows, np.ones(3) / 3)
    idx = [inputs.draw_ids(rng, vocab, 1.0, int(k)) for k in sizes]
    val = [inputs.small_integer_values(rng, (int(k), dim)) for k in sizes]
    table = (rng.standard_normal((vocab, dim)) * 0.02).astype(np.float32)
    run_chain(gpu, idx, val, dim, vocab, 16, "mod", "sgd", 0.5, table, check_rows_exact=True)


def test_unaligned_value_pointers(gpu):
    """Value rows that start 4 bytes into an allocation take the element-wise path."""
    ctx, px, runner = gpu
    rng = np.random.default_rng(3)
    dim, vocab = 64, 200
    idx = [rng.integers(0, vocab, size=300, dtype=np.int64) for _ in range(2)]
    val = [rng.standard_normal((300, dim), dtype=np.float32) for _ in range(2)]
    d_idx = [runner.to_device(i) for i in idx]
    backing = [torch.empty(300 * dim + 1, dtype=torch.float32, device="cuda") for _ in range(2)]
    d_val = []
    for bk, v in zip(backing, val):
        bk[1:].copy_(torch.from_numpy(v).reshape(-1))
        d_val.append(bk[1:])
        assert d_val[-1].data_ptr() % 16 == 4
    b = runner.sparse_buffers(d_idx, d_val, dim, vocab, 2, px.PX_HASH_MOD)
    runner.coalesce(ctx, b)
    u = int(b.out_num.item())
    o_ids, o_rows, _ = oracle.sparse_coalesce(idx, val, dim, vocab)
    assert np.array_equal(b.out_ids[:u].cpu().numpy(), o_ids)
    close(b.out_rows[:u].cpu().numpy(), o_rows)


# ---------------------------------------------------------------- edge cases

def test_empty_input(gpu):
    ctx, px, runner = gpu
    dim, vocab = 16, 100
    e_i = torch.zeros(0, dtype=torch.int64, device="cuda")
    e_v = torch.zeros((0, dim), dtype=torch.float32, device="cuda")
    b = runner.sparse_buffers([e_i, e_i], [e_v, e_v], dim, vocab, 4, px.PX_HASH_MUL)
    b.out_num.fill_(77)
    table = torch.randn(vocab, dim, device="cuda")
    before = table.clone()
    runner.sparse_step(ctx, b, table, None, "sgd", 0.5)
    assert int(b.out_num.item()) == 0
    assert np.array_equal(b.offsets.cpu().numpy(), np.zeros(5, dtype=np.int64))
    assert torch.equal(table, before)


def test_ragged_workers_with_an_empty_one(gpu):
    rng = np.random.default_rng(4)
    dim, vocab = 32, 1000
    sizes = [0, 1, 2047, 0, 2049, 5]
    idx = [rng.integers(0, vocab, size=n, dtype=np.int64) for n in sizes]
    val = [rng.standard_normal((n, dim), dtype=np.float32) for n in sizes]
    table = np.zeros((vocab, dim), dtype=np.float32)
    run_chain(gpu, idx, val, dim, vocab, 7, "mod", "sgd", 1.0, table)


def test_most_workers_allowed(gpu):
    """PX_MAX_SOURCES workers (the pointer tables take several uploads), a few rows each."""
    ctx, px, runner = gpu
    rng = np.random.default_rng(44)
    dim, vocab, n = 16, 700, px.PX_MAX_SOURCES
    sizes = rng.integers(0, 6, size=n)
    idx = [rng.integers(0, vocab, size=int(k), dtype=np.int64) for k in sizes]
    val = [rng.standard_normal((int(k), dim), dtype=np.float32) for k in sizes]
    table = np.zeros((vocab, dim), dtype=np.float32)
    run_chain(gpu, idx, val, dim, vocab, 16, "mul", "sgd", 0.3, table)
    with pytest.raises(px.PxError) as e:
        b = runner.sparse_buffers([runner.to_device(idx[0])] * (n + 1), [runner.to_device(val[0])] * (n + 1), dim,
                                  vocab, 2, px.PX_HASH_MOD)
        runner.coalesce(ctx, b)
    assert e.value.status == px.PX_ERR_INVALID_ARG


def test_single_worker_all_distinct_is_a_permutation(gpu):
    rng = np.random.default_rng(5)
    dim, vocab = 48, 6000
    ids = rng.permutation(vocab)[:5000].astype(np.int64)
    val = rng.standard_normal((5000, dim), dtype=np.float32)
    table = np.zeros((vocab, dim), dtype=np.float32)
    run_chain(gpu, [ids], [val], dim, vocab, 2, "mod", "sgd", 1.0, table, check_rows_exact=True)


def test_all_rows_share_one_id(gpu):
    """One run through every tile: the border-crossing path end to end."""
    rng = np.random.default_rng(6)
    dim, vocab = 128, 50
    idx = [np.full(3000, 17, dtype=np.int64) for _ in range(4)]
    val = [rng.standard_normal((3000, dim), dtype=np.float32) for _ in range(4)]
    table = np.zeros((vocab, dim), dtype=np.float32)
    b, u = run_chain(gpu, idx, val, dim, vocab, 4, "mul", "sgd", 0.01, table)
    assert u == 1


def test_integer_valued_rows_are_bit_exact(gpu):
    rng = np.random.default_rng(7)
    dim, vocab = 256, 300
    idx = [inputs.draw_ids(rng, vocab, 1.3, 6000) for _ in range(6)]
    val = [inputs.small_integer_values(rng, (6000, dim)) for _ in range(6)]
    table = np.zeros((vocab, dim), dtype=np.float32)
    run_chain(gpu, idx, val, dim, vocab, 8, "mul", "sgd", 1.0, table, check_rows_exact=True)


def test_average_scale(gpu):
    rng = np.random.default_rng(8)
    dim, vocab, n = 64, 400, 8
    idx = [inputs.draw_ids(rng, vocab, 1.0, 500) for _ in range(n)]
    val = [rng.standard_normal((500, dim), dtype=np.float32) for _ in range(n)]
    table = np.zeros((vocab, dim), dtype=np.float32)
    run_chain(gpu, idx, val, dim, vocab, 4, "mul", "sgd", 0.1, table, scale=1.0 / n)


def test_vocab_of_one_and_of_two_to_the_32(gpu):
    ctx, px, runner = gpu
    rng = np.random.default_rng(9)
    dim = 8
    val = [rng.standard_normal((100, dim), dtype=np.float32)]
    table = np.zeros((1, dim), dtype=np.float32)
    run_chain(gpu, [np.zeros(100, dtype=np.int64)], val, dim, 1, 1, "mod", "sgd", 1.0, table)
    # ids that need all 32 key bits (coalesce and partition only: no table that large)
    vocab = 1 << 32
    ids = np.concatenate([rng.integers(vocab - 1000, vocab, size=60, dtype=np.int64),
                          rng.integers(0, 1000, size=40, dtype=np.int64)])
    b = runner.sparse_buffers([runner.to_device(ids)], [runner.to_device(val[0])], dim, vocab, 5,
                              px.PX_HASH_MUL)
    runner.coalesce(ctx, b)
    runner.partition(ctx, b)
    u = int(b.out_num.item())
    o_ids, o_rows, _ = oracle.sparse_coalesce([ids], val, dim, vocab)
    assert np.array_equal(b.out_ids[:u].cpu().numpy(), o_ids)
    close(b.out_rows[:u].cpu().numpy(), o_rows)
    o_shard, o_perm, o_off = oracle.partition_rows(o_ids, 5, "mul")
    assert np.array_equal(b.shard[:u].cpu().numpy(), o_shard)
    assert np.array_equal(b.perm[:u].cpu().numpy(), o_perm)
    assert np.array_equal(b.offsets.cpu().numpy(), o_off)


def test_two_runs_give_the_same_bits(gpu):
    ctx, px, runner = gpu
    w = inputs.shrink(inputs.STRESS_ZIPF, vocab=100_000, n_workers=8, n_per_worker=5000)
    d_idx = [runner.to_device(i) for i in inputs.sparse_ids(w)]
    d_val = [runner.to_device(v) for v in inputs.sparse_values(w)]
    outs = []
    for _ in range(2):
        b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, px.PX_HASH_MUL)
        runner.coalesce(ctx, b)
        runner.partition(ctx, b)
        u = int(b.out_num.item())
        outs.append((b.out_ids[:u].clone(), b.out_rows[:u].clone(), b.perm[:u].clone()))
    assert all(torch.equal(x, y) for x, y in zip(*outs))


def test_out_of_range_id_raises_the_flag_and_protects_the_table(gpu):
    ctx, px, runner = gpu
    dim, vocab = 16, 100
    for bad in (-1, vocab, 1 << 40):
        ids = torch.tensor([3, 5, bad, 7], dtype=torch.int64, device="cuda")
        val = torch.ones((4, dim), dtype=torch.float32, device="cuda")
        b = runner.sparse_buffers([ids], [val], dim, vocab, 2, px.PX_HASH_MOD)
        table = torch.randn(vocab, dim, device="cuda")
        before = table.clone()
        runner.sparse_step(ctx, b, table, None, "sgd", 0.5)
        assert int(b.out_num.item()) == 0
        assert torch.equal(table, before)
        assert ctx.px_device_status() == px.PX_ERR_INDEX_OUT_OF_RANGE
        assert ctx.px_device_status() == px.PX_OK          # reported once, then cleared
        accum = torch.ones_like(table)
        runner.fused_step(ctx, b, table, accum, "adagrad", 0.5)
        assert int(b.out_num.item()) == 0
        assert torch.equal(table, before) and bool((accum == 1).all())
        assert ctx.px_device_status() == px.PX_ERR_INDEX_OUT_OF_RANGE
    # apply checks the ids it is handed as well
    ids = torch.tensor([1, vocab + 5], dtype=torch.int64, device="cuda")
    rows = torch.ones((2, dim), dtype=torch.float32, device="cuda")
    num = torch.tensor([2], dtype=torch.int64, device="cuda")
    table = torch.zeros(vocab, dim, device="cuda")
    ctx.px_sparse_apply_sgd(table, ids, rows, num, 2, None, None, 1.0)
    assert ctx.px_device_status() == px.PX_ERR_INDEX_OUT_OF_RANGE
    assert float(table[1, 0]) == -1.0 and float(table.abs().sum()) == dim


def test_repeated_id_in_apply_is_reported_and_its_row_left_alone(gpu):
    """Sec. 2.1: gradients are aggregated first, so that a row is updated once.  An id that repeats
    (adjacent, as in any sorted list) is refused by the oracle; the library skips exactly those
    positions, updates the others, and reports PX_ERR_NOT_UNIQUE once."""
    ctx, px, runner = gpu
    dim, vocab = 24, 50
    rng = np.random.default_rng(17)
    ids = np.array([2, 7, 7, 9, 20, 20, 20, 31], dtype=np.int64)
    rows = rng.standard_normal((ids.size, dim)).astype(np.float32)
    table = rng.standard_normal((vocab, dim)).astype(np.float32)
    with pytest.raises(oracle.RepeatedId):
        oracle.sparse_apply_sgd(table.copy(), ids, rows, 0.5)
    keep = np.array([0, 3, 7])                                   # the positions whose id occurs once
    for optimizer in ("sgd", "adagrad"):
        ref_t, ref_a = table.copy(), np.full_like(table, 0.1)
        d_t, d_a = torch.from_numpy(table).cuda(), torch.full((vocab, dim), 0.1, device="cuda")
        num = torch.tensor([ids.size], dtype=torch.int64, device="cuda")
        if optimizer == "sgd":
            oracle.sparse_apply_sgd(ref_t, ids[keep], rows[keep], 0.5)
            ctx.px_sparse_apply_sgd(d_t, runner.to_device(ids), runner.to_device(rows), num, ids.size, None, None, 0.5)
        else:
            oracle.sparse_apply_adagrad(ref_t, ref_a, ids[keep], rows[keep], 0.5)
            ctx.px_sparse_apply_adagrad(d_t, d_a, runner.to_device(ids), runner.to_device(rows), num, ids.size,
                                        None, None, 0.5)
        assert ctx.px_device_status() == px.PX_ERR_NOT_UNIQUE
        assert ctx.px_device_status() == px.PX_OK                # reported once, then cleared
        close(d_t.cpu().numpy(), ref_t)
        close(d_a.cpu().numpy(), ref_a)
        for r in (7, 20):                                        # the repeated ids' rows: bit-identical
            assert np.array_equal(d_t[r].cpu().numpy(), table[r])
    # while the flag is up, later updates on the context leave their table alone
    ids2 = torch.tensor([1, 1, 4], dtype=torch.int64, device="cuda")
    rows2 = torch.ones((3, dim), device="cuda")
    num2 = torch.tensor([3], dtype=torch.int64, device="cuda")
    t2 = torch.zeros((vocab, dim), device="cuda")
    ctx.px_sparse_apply_sgd(t2, ids2, rows2, num2, 3, None, None, 1.0)
    ids3 = torch.tensor([5, 6], dtype=torch.int64, device="cuda")
    ctx.px_sparse_apply_sgd(t2, ids3, rows2, torch.tensor([2], dtype=torch.int64, device="cuda"), 2, None, None, 1.0)
    assert float(t2[4, 0]) == -1.0 and float(t2.abs().sum()) == dim        # only id 4 of the first call
    assert ctx.px_device_status() == px.PX_ERR_NOT_UNIQUE
    # distinct ids in any order are fine, and so is the last position equalling nothing
    ids4 = np.array([40, 3, 12, 11], dtype=np.int64)
    t4 = torch.zeros((vocab, dim), device="cuda")
    ctx.px_sparse_apply_sgd(t4, runner.to_device(ids4), torch.ones((4, dim), device="cuda"),
                            torch.tensor([4], dtype=torch.int64, device="cuda"), 4, None, None, 1.0)
    assert ctx.px_device_status() == px.PX_OK and float(t4.sum()) == -4.0 * dim


def test_a_given_up_wait_is_reported_and_harmless(gpu):
    """The head ranking and the one-launch partition let a workgroup wait, for a bounded number of
    polls, for counts other workgroups publish.  With the limit at 0 every wait that is not already
    satisfied is given up: the call must still end normally, touch nothing out of bounds, leave the
    table alone and report PX_ERR_DEVICE (or, if no workgroup ever had to wait, give the right
    result); with the limit restored the same context works again."""
    _, px, runner = gpu
    ctx = px.Context(0)
    with pytest.raises(px.PxError):
        ctx.px_set_wait_limit(-1)
    w = inputs.shrink(inputs.LARGE_LM, vocab=50_000, n_per_worker=2_000, dim=64)     # 96,000 rows: 94 sort blocks
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    table = inputs.table_init(w)
    accum = inputs.accum_init(w)
    d_idx = [runner.to_device(i) for i in idx]
    d_val = [runner.to_device(v) for v in val]
    o_ids, o_rows, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab)
    _, o_perm, o_off = oracle.partition_rows(o_ids, w.n_shards, "mul")
    ref_t, ref_a = table.copy(), accum.copy()
    oracle.sparse_apply_adagrad(ref_t, ref_a, o_ids, o_rows, w.lr, perm=o_perm)
    seen = set()
    for limit in (0, 0, 0, 1 << 18):
        ctx.px_set_wait_limit(limit)
        b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, px.PX_HASH_MUL)
        d_t, d_a = torch.from_numpy(table).cuda(), torch.from_numpy(accum).cuda()
        runner.sparse_step(ctx, b, d_t, d_a, "adagrad", w.lr)
        status = ctx.px_device_status()
        seen.add(status)
        assert status in (px.PX_OK, px.PX_ERR_DEVICE)
        if limit:
            assert status == px.PX_OK
        if status == px.PX_ERR_DEVICE:
            assert np.array_equal(d_t.cpu().numpy(), table) and np.array_equal(d_a.cpu().numpy(), accum)
            assert 0 <= int(b.out_num.item()) <= o_ids.size
        else:
            u = int(b.out_num.item())
            assert u == o_ids.size and np.array_equal(b.out_ids[:u].cpu().numpy(), o_ids)
            assert np.array_equal(b.perm[:u].cpu().numpy(), o_perm) and np.array_equal(b.offsets.cpu().numpy(), o_off)
            close(b.out_rows[:u].cpu().numpy(), o_rows)
            close(d_t.cpu().numpy()[o_ids], ref_t[o_ids])
            close(d_a.cpu().numpy()[o_ids], ref_a[o_ids])
        assert ctx.px_device_status() == px.PX_OK                  # reported once, then cleared
    assert px.PX_OK in seen
    ctx.close()


def test_host_side_argument_errors(gpu):
    ctx, px, runner = gpu
    dim, vocab = 16, 100
    ids = torch.zeros(10, dtype=torch.int64, device="cuda")
    val = torch.zeros((10, dim), dtype=torch.float32, device="cuda")
    b = runner.sparse_buffers([ids], [val], dim, vocab, 2, px.PX_HASH_MOD)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(px.PxError) as e:
        ctx.px_sparse_coalesce(b.idx, b.val, dim, vocab, 1.0, b.out_ids, b.out_rows, b.out_num, None, small)
    assert e.value.status == px.PX_ERR_SCRATCH_TOO_SMALL
    with pytest.raises(px.PxError) as e:
        ctx.px_sparse_coalesce(b.idx, b.val, dim, 0, 1.0, b.out_ids, b.out_rows, b.out_num, None, b.scratch)
    assert e.value.status == px.PX_ERR_INVALID_ARG
    with pytest.raises(px.PxError) as e:
        ctx.px_partition_rows(b.out_ids, b.out_num, 10, px.PX_MAX_SHARDS + 1, px.PX_HASH_MOD, None, b.perm,
                              b.offsets, b.part_scratch)
    assert e.value.status == px.PX_ERR_INVALID_ARG


def test_two_level_aggregation(gpu):
    """Local aggregation per machine, then global (Sec. 4.3): 8 groups of 6 workers, as in the paper's
    cluster.  Same ids; rows equal the one-level result up to the float rounding of the group sums,
    and equal the oracle run the same two-level way to the last bit or so."""
    ctx, px, runner = gpu
    w = inputs.shrink(inputs.LARGE_LM, vocab=60_000, n_per_worker=700)
    idx, val = inputs.sparse_ids(w), inputs.sparse_values(w)
    d_idx = [runner.to_device(i) for i in idx]
    d_val = [runner.to_device(v) for v in val]
    second, firsts = runner.two_level_coalesce(ctx, d_idx, d_val, w.dim, w.vocab, 6)
    assert len(firsts) == 8 and ctx.px_device_status() == px.PX_OK
    u = int(second.out_num.item())
    o_ids, o_rows, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab)
    assert u == o_ids.size and np.array_equal(second.out_ids[:u].cpu().numpy(), o_ids)
    # against the one-level sum: each of the 8 group sums was rounded to float (half an ulp of a value
    # of magnitude up to ~100, i.e. ~4e-6) before the second level, so sums that cancel keep that error
    close(second.out_rows[:u].cpu().numpy(), o_rows, abs_=8 * 4e-6)
    gi, gv = [], []
    for g in range(8):
        a, b, _ = oracle.sparse_coalesce(idx[6 * g:6 * g + 6], val[6 * g:6 * g + 6], w.dim, w.vocab)
        gi.append(a)
        gv.append(b)
        n = int(firsts[g].out_num.item())
        assert np.array_equal(firsts[g].out_ids[:n].cpu().numpy(), a)
    t_ids, t_rows, _ = oracle.sparse_coalesce(gi, gv, w.dim, w.vocab)
    x, ref = second.out_rows[:u].cpu().numpy(), t_rows
    assert np.all(np.abs(x - ref) <= 2 * np.spacing(np.abs(ref)))


def test_partition_search_on_measured_chain_times(gpu):
    """Sec. 3.2, Eq. 1 on this machine: the library's sampling rule is driven by times of the sparse
    chain measured on the device; the recorded (P, time) list is then handed to the oracle, which
    must visit the same partition counts in the same order, fit the same theta and pick the same P."""
    import cost_model_checks
    ctx, px, runner = gpu
    from oracle import cost_model
    w = inputs.shrink(inputs.LARGE_LM, vocab=200_000, n_per_worker=1_000)
    d_idx = [runner.to_device(i) for i in inputs.sparse_ids(w)]
    d_val = [runner.to_device(v) for v in inputs.sparse_values(w)]
    table = torch.zeros((w.vocab, w.dim), device="cuda")
    accum = torch.full((w.vocab, w.dim), w.accum_init, device="cuda")

    def measure(n_shards):
        b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, n_shards, px.PX_HASH_MUL)
        times = []
        for it in range(8):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            runner.sparse_step(ctx, b, table, accum, w.optimizer, w.lr)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
        return float(np.median(times[2:]))

    for start, p_max in ((8, 256), (2, 16)):
        ps, ts = [], []
        while True:
            nxt = px.px_partition_search_next(ps, ts, start, p_max)
            if nxt == 0:
                break
            assert nxt not in ps and 1 <= nxt <= p_max and len(ps) < 16
            ps.append(nxt)
            ts.append(measure(nxt))
        cost_model_checks.check_recorded_search(px, cost_model, ps, ts, start, p_max)
    assert ctx.px_device_status() == px.PX_OK


def test_cost_model_library_against_the_oracle_on_this_box():
    """The host-only comparisons of the cost model, collected by the GPU run as well (they need no
    device, but the library they load is the one the GPU tests use)."""
    import test_cost_model
    from paper_1808_02621_amd import px
    test_cost_model.test_library_fit_and_argmin_match_the_oracle(px)
    test_cost_model.test_library_search_follows_the_same_samples(px)
    for p in ([3, 7, 3, 7], [8, 16, 16, 8, 8]):
        test_cost_model.test_library_fit_rejects_two_distinct_partition_counts(px, p)


def test_whole_path_replays_from_a_hip_graph(gpu):
    """The calls only enqueue kernels (no allocation, no memset, no host staging), so the whole path can
    be captured once and replayed; every replay, with fresh inputs written into the same buffers and
    eager work in between, must give the eager result."""
    ctx, px, runner = gpu
    w = inputs.shrink(inputs.LARGE_LM, vocab=30_000, n_workers=8, n_per_worker=1500, dim=128, dense_count=50_000)
    rng = np.random.default_rng(77)

    def fresh():
        idx = [inputs.draw_ids(rng, w.vocab, 1.0, w.n_per_worker) for _ in range(w.n_workers)]
        val = [rng.standard_normal((w.n_per_worker, w.dim), dtype=np.float32) for _ in range(w.n_workers)]
        dense = [rng.standard_normal(w.dense_count, dtype=np.float32) for _ in range(w.n_workers)]
        return idx, val, dense

    idx, val, dense = fresh()
    d_idx = [runner.to_device(i) for i in idx]
    d_val = [runner.to_device(v) for v in val]
    d_dense = [runner.to_device(x) for x in dense]
    b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, px.PX_HASH_MUL)
    table0 = torch.from_numpy(inputs.table_init(w)).cuda()
    accum0 = torch.from_numpy(inputs.accum_init(w)).cuda()
    table, accum = table0.clone(), accum0.clone()
    f_table, f_accum = table0.clone(), accum0.clone()
    dense_out = torch.empty(w.dense_count, dtype=torch.float32, device="cuda")
    pulled = torch.empty((w.total_rows, w.dim), dtype=torch.float32, device="cuda")
    all_ids = torch.cat(d_idx)

    def whole_path(t, a):
        runner.sparse_step(ctx, b, t, a, "adagrad", w.lr)
        ctx.px_dense_average(d_dense, w.dense_count, dense_out, 1.0 / w.n_workers)
        ctx.px_sparse_lookup(t, all_ids, None, w.total_rows, None, None, pulled)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        whole_path(table, accum)                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    table.copy_(table0)
    accum.copy_(accum0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        whole_path(table, accum)
    table.copy_(table0)                                            # capture does not run anything
    accum.copy_(accum0)

    for replay in range(4):
        if replay:
            idx, val, dense = fresh()
            for dst, src in zip(d_idx, idx):
                dst.copy_(torch.from_numpy(src))
            for dst, src in zip(d_val, val):
                dst.copy_(torch.from_numpy(src))
            for dst, src in zip(d_dense, dense):
                dst.copy_(torch.from_numpy(src))
            all_ids.copy_(torch.cat(d_idx))
        graph.replay()
        torch.cuda.synchronize()
        got = (table.clone(), accum.clone(), dense_out.clone(), pulled.clone(), b.out_ids.clone(), int(b.out_num.item()),
               b.perm.clone(), b.offsets.clone(), b.shard.clone())
        whole_path(f_table, f_accum)                               # the same step, eagerly, on the twin state
        torch.cuda.synchronize()
        assert ctx.px_device_status() == px.PX_OK
        u = int(b.out_num.item())
        assert got[5] == u and torch.equal(got[4][:u], b.out_ids[:u])
        assert torch.equal(got[6][:u], b.perm[:u]) and torch.equal(got[7], b.offsets) and torch.equal(got[8][:u], b.shard[:u])
        assert torch.equal(got[0], f_table) and torch.equal(got[1], f_accum)
        assert torch.equal(got[2], dense_out) and torch.equal(got[3], pulled)
    ref_ids, _, _ = oracle.sparse_coalesce(idx, val, w.dim, w.vocab)
    assert np.array_equal(b.out_ids[:u].cpu().numpy(), ref_ids)
    assert not torch.equal(f_table, table0)
    # three replays in a row, new ids before each, nothing eager in between: whatever a replay leaves
    # behind in scratch or in the context must not leak into the next one
    for _ in range(3):
        idx, val, dense = fresh()
        for dst, src in zip(d_idx, idx):
            dst.copy_(torch.from_numpy(src))
        graph.replay()
    torch.cuda.synchronize()
    assert ctx.px_device_status() == px.PX_OK
    ref_ids, _, ref_len = oracle.sparse_coalesce(idx, [np.zeros((w.n_per_worker, w.dim), np.float32)] * w.n_workers, w.dim, w.vocab)
    u = int(b.out_num.item())
    assert u == ref_ids.size and np.array_equal(b.out_ids[:u].cpu().numpy(), ref_ids)
    assert np.array_equal(b.out_run_len[:u].cpu().numpy(), ref_len)
    o_shard, o_perm, o_off = oracle.partition_rows(ref_ids, w.n_shards, "mul")
    assert np.array_equal(b.shard[:u].cpu().numpy(), o_shard) and np.array_equal(b.perm[:u].cpu().numpy(), o_perm)
    assert np.array_equal(b.offsets.cpu().numpy(), o_off)


# ---------------------------------------------------------------- partition

@pytest.mark.parametrize("n_shards", [1, 2, 3, 7, 16, 100, 256])
@pytest.mark.parametrize("hash_name", ["mod", "mul"])
def test_partition_shard_counts(gpu, n_shards, hash_name):
    ctx, px, runner = gpu
    rng = np.random.default_rng(n_shards)
    ids = np.unique(rng.integers(0, 1 << 31, size=9000, dtype=np.int64))
    cap = ids.size + 500                                   # capacity larger than the real count
    d_ids = torch.zeros(cap, dtype=torch.int64, device="cuda")
    d_ids[:ids.size] = torch.from_numpy(ids).cuda()
    d_ids[ids.size:] = -12345                              # must never be looked at
    num = torch.tensor([ids.size], dtype=torch.int64, device="cuda")
    shard = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    perm = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    off = torch.empty(n_shards + 1, dtype=torch.int64, device="cuda")
    scratch = px.alloc_scratch(px.Context.px_partition_scratch_bytes(cap))
    code = px.PX_HASH_MUL if hash_name == "mul" else px.PX_HASH_MOD
    ctx.px_partition_rows(d_ids, num, cap, n_shards, code, shard, perm, off, scratch)
    o_shard, o_perm, o_off = oracle.partition_rows(ids, n_shards, hash_name)
    assert np.array_equal(shard[:ids.size].cpu().numpy(), o_shard)
    assert np.array_equal(perm[:ids.size].cpu().numpy(), o_perm)
    assert np.array_equal(off.cpu().numpy(), o_off)
    assert bool((shard[ids.size:] == -1).all()) and bool((perm[ids.size:] == -1).all())


@pytest.mark.parametrize("cap,n_shards", [(1023, 5), (1024, 256), (1025, 2), (2047, 3), (2048, 256), (2049, 8), (524_288, 4), (524_289, 4), (60_000, 8), (60_000, 64), (60_000, 70),
                                          (131_072, 32), (131_072, 33), (400_000, 10), (400_000, 11), (1_100_000, 1),
                                          (1_100_000, 16)])
def test_partition_one_launch_and_two_launch_paths(gpu, cap, n_shards):
    """A partition of few blocks x shards runs as one launch whose blocks exchange their shard counts,
    a larger one as histogram (, prefix) and scatter launches: both sides of every switch, several
    calls in a row on one context (the exchanged counts are told apart by the call's number), a count
    well below the capacity, a full one and an empty one."""
    ctx, px, runner = gpu
    rng = np.random.default_rng(cap + n_shards)
    scratch = px.alloc_scratch(px.Context.px_partition_scratch_bytes(cap))
    d_ids = torch.empty(cap, dtype=torch.int64, device="cuda")
    for n in (cap, max(1, cap // 3), 0, min(cap, 5)):
        ids = np.unique(rng.integers(0, 1 << 40, size=n, dtype=np.int64))[:n]
        hash_name = "mul" if n % 2 else "mod"
        d_ids.fill_(-999)
        d_ids[:ids.size] = torch.from_numpy(ids).cuda()
        num = torch.tensor([ids.size], dtype=torch.int64, device="cuda")
        shard = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        perm = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        off = torch.full((n_shards + 1,), -1, dtype=torch.int64, device="cuda")
        ctx.px_partition_rows(d_ids, num, cap, n_shards, px.PX_HASH_MUL if hash_name == "mul" else px.PX_HASH_MOD,
                              shard, perm, off, scratch)
        o_shard, o_perm, o_off = oracle.partition_rows(ids, n_shards, hash_name)
        assert np.array_equal(off.cpu().numpy(), o_off)
        assert np.array_equal(shard[:ids.size].cpu().numpy(), o_shard)
        assert np.array_equal(perm[:ids.size].cpu().numpy(), o_perm)
        assert bool((shard[ids.size:] == -1).all()) and bool((perm[ids.size:] == -1).all())
    assert ctx.px_device_status() == px.PX_OK


def test_apply_shard_by_shard_equals_apply_all(gpu):
    ctx, px, runner = gpu
    w = inputs.shrink(inputs.LARGE_LM, vocab=20_000, n_workers=8, n_per_worker=1000, dim=64)
    d_idx = [runner.to_device(i) for i in inputs.sparse_ids(w)]
    d_val = [runner.to_device(v) for v in inputs.sparse_values(w)]
    b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, px.PX_HASH_MUL)
    runner.coalesce(ctx, b)
    runner.partition(ctx, b)
    t0 = torch.from_numpy(inputs.table_init(w)).cuda()
    a0 = torch.from_numpy(inputs.accum_init(w)).cuda()
    t_all, a_all = t0.clone(), a0.clone()
    runner.apply(ctx, b, t_all, a_all, "adagrad", w.lr)
    t_sh, a_sh = t0.clone(), a0.clone()
    for p in range(w.n_shards):
        runner.apply(ctx, b, t_sh, a_sh, "adagrad", w.lr, range_=b.offsets[p:p + 2])
    assert torch.equal(t_all, t_sh) and torch.equal(a_all, a_sh)
    assert not torch.equal(t_all, t0)
    # one shard alone touches only ids of that shard
    t_one = t0.clone()
    runner.apply(ctx, b, t_one, a0.clone(), "adagrad", w.lr, range_=b.offsets[2:4])
    changed = (t_one != t0).any(dim=1).nonzero().flatten().cpu().numpy()
    assert changed.size > 0
    assert all(((int(c) * 2654435761) % (1 << 64)) % w.n_shards == 2 for c in changed)


# -------------------------------------------------------------------- lookup

@pytest.mark.parametrize("dim", [1, 6, 64, 100, 128, 512, 1024, 1300])
def test_lookup_stitches_shards_in_batch_order(gpu, dim):
    ctx, px, runner = gpu
    rng = np.random.default_rng(dim)
    vocab, n, p = 3000, 5000, 8
    table = rng.standard_normal((vocab, dim), dtype=np.float32)
    ids = inputs.draw_ids(rng, vocab, 1.1, n)                         # a batch repeats words
    d_table, d_ids = torch.from_numpy(table).cuda(), torch.from_numpy(ids).cuda()
    out = torch.full((n, dim), float("nan"), device="cuda")
    ctx.px_sparse_lookup(d_table, d_ids, None, n, None, None, out)
    assert np.array_equal(out.cpu().numpy(), oracle.sparse_lookup(table, ids))
    # per shard, then stitched: partition the batch ids, pull every shard's rows into place
    num = torch.tensor([n], dtype=torch.int64, device="cuda")
    perm = torch.empty(n, dtype=torch.int32, device="cuda")
    off = torch.empty(p + 1, dtype=torch.int64, device="cuda")
    ctx.px_partition_rows(d_ids, num, n, p, px.PX_HASH_MUL, None, perm, off,
                          px.alloc_scratch(px.Context.px_partition_scratch_bytes(n)))
    o_shard, o_perm, o_off = oracle.partition_rows(ids, p, "mul")
    assert np.array_equal(perm.cpu().numpy(), o_perm) and np.array_equal(off.cpu().numpy(), o_off)
    stitched = torch.full((n, dim), float("nan"), device="cuda")
    ref = np.full((n, dim), np.nan, dtype=np.float32)
    for q in range(p):
        ctx.px_sparse_lookup(d_table, d_ids, num, n, perm, off[q:q + 2], stitched)
        oracle.sparse_lookup(table, ids, perm=o_perm, first=int(o_off[q]), last=int(o_off[q + 1]), out=ref)
        assert np.array_equal(stitched.cpu().numpy(), ref, equal_nan=True)
    assert torch.equal(stitched, out)
    assert ctx.px_device_status() == px.PX_OK


def test_lookup_full_size_and_bad_id(gpu):
    ctx, px, runner = gpu
    w = inputs.NMT
    table = inputs.table_init(w)
    ids = np.concatenate(inputs.sparse_ids(w))                       # all 48 workers' pulls of one table
    d_table, d_ids = torch.from_numpy(table).cuda(), torch.from_numpy(ids).cuda()
    out = torch.empty((ids.size, w.dim), device="cuda")
    ctx.px_sparse_lookup(d_table, d_ids, None, ids.size, None, None, out)
    assert np.array_equal(out.cpu().numpy(), oracle.sparse_lookup(table, ids))
    bad = torch.tensor([5, w.vocab, 7], dtype=torch.int64, device="cuda")
    out3 = torch.full((3, w.dim), -1.0, device="cuda")
    ctx.px_sparse_lookup(d_table, bad, None, 3, None, None, out3)
    assert ctx.px_device_status() == px.PX_ERR_INDEX_OUT_OF_RANGE
    assert torch.equal(out3[0], d_table[5]) and torch.equal(out3[2], d_table[7]) and bool((out3[1] == -1).all())


# --------------------------------------------------------------------- dense

@pytest.mark.parametrize("n_buffers,count", [(1, 1000), (4, 65_536), (8, 4099), (48, 70_001), (65, 513),
                                             (300, 2048)])
@pytest.mark.parametrize("bf16", [False, True])
def test_dense_average(gpu, n_buffers, count, bf16):
    ctx, px, runner = gpu
    rng = np.random.default_rng(n_buffers + count)
    bufs = [rng.standard_normal(count, dtype=np.float32) for _ in range(n_buffers)]
    if bf16:
        bufs = [inputs.f32_to_bf16_bits(b) for b in bufs]
    d = [runner.to_device(b) for b in bufs]
    out = torch.empty(count, dtype=torch.float32, device="cuda")
    ctx.px_dense_average(d, count, out, 1.0 / n_buffers)
    close(out.cpu().numpy(), oracle.dense_average(bufs, average=True))
    ctx.px_dense_average(d, count, out, 1.0)
    close(out.cpu().numpy(), oracle.dense_average(bufs, average=False))
    if n_buffers == 1 and not bf16:
        assert np.array_equal(out.cpu().numpy(), bufs[0])


@pytest.mark.parametrize("bf16", [False, True])
def test_dense_average_over_several_launches_with_a_ragged_tail(gpu, bf16):
    """Two buffers: a launch covers 16 MiB of output, so this count takes two launches (the second one
    partly filled, its last workgroup ragged) plus the element-wise tail; integer values, bit-exact."""
    ctx, px, runner = gpu
    count = 6_300_003
    assert px.px_dense_average_launches(2, count, bf16) == 2
    rng = np.random.default_rng(5 + int(bf16))
    bufs = [inputs.small_integer_values(rng, count) for _ in range(2)]
    if bf16:
        bufs = [inputs.f32_to_bf16_bits(b) for b in bufs]
    d = [runner.to_device(b) for b in bufs]
    out = torch.full((count + 8,), float("nan"), dtype=torch.float32, device="cuda")
    ctx.px_dense_average(d, count, out, 1.0)
    assert np.array_equal(out[:count].cpu().numpy(), oracle.dense_average(bufs, average=False))
    assert bool(torch.isnan(out[count:]).all())                        # nothing written past the end
    ctx.px_dense_average(d, count, out, 0.5)
    assert np.array_equal(out[:count].cpu().numpy(), oracle.dense_average(bufs, average=True))


@pytest.mark.parametrize("seed", range(24))
def test_dense_average_random_cases(gpu, seed):
    """Random buffer counts, lengths, element types, output types and alignments; nothing written past the end."""
    ctx, px, runner = gpu
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.choice([1, 2, 3, 5, 8, 17, 48, 64, 90]))
    count = int(rng.choice([1, 7, 255, 1024, 4097, 65_537, 300_001, 1_048_576 + 13, 2_500_000]))
    count = min(count, 30_000_000 // n)
    bf16 = bool(rng.integers(0, 2))
    out_bf16 = bool(rng.integers(0, 4) == 0)
    off = int(rng.choice([0, 0, 0, 1, 4]))                        # elements into the allocation: alignment
    bufs = [rng.standard_normal(count + off, dtype=np.float32) for _ in range(n)]
    if bf16:
        bufs = [inputs.f32_to_bf16_bits(b) for b in bufs]
    d = [runner.to_device(b)[off:] for b in bufs]
    out = torch.full((count + 4,), 7.0, dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda")
    scale = float(rng.choice([1.0, 1.0 / n]))
    ctx.px_dense_average(d, count, out, scale)
    ref = oracle.dense_average([b[off:] for b in bufs], average=(scale != 1.0))
    close(out[:count].float().cpu().numpy(), ref, 1e-2 if out_bf16 else REL_TOL)
    assert bool((out[count:].float() == 7.0).all())


def test_dense_average_bf16_output_and_unaligned(gpu):
    ctx, px, runner = gpu
    rng = np.random.default_rng(21)
    count, n = 5001, 6
    bufs = [rng.standard_normal(count + 1, dtype=np.float32) for _ in range(n)]
    d = [runner.to_device(b) for b in bufs]
    ref = oracle.dense_average([b[1:] for b in bufs], average=True)
    out = torch.empty(count, dtype=torch.float32, device="cuda")
    ctx.px_dense_average([x[1:] for x in d], count, out, 1.0 / n)          # 4-byte aligned only
    close(out.cpu().numpy(), ref)
    out16 = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    ctx.px_dense_average([x[1:] for x in d], count, out16, 1.0 / n)
    ref16 = torch.from_numpy(ref).to(torch.bfloat16)
    assert torch.equal(out16.cpu(), ref16)
    aligned = [x[:count - 1].contiguous() for x in d]
    ctx.px_dense_average(aligned, count - 1, out16, 1.0 / n)
    ref16 = torch.from_numpy(oracle.dense_average([b[:count - 1] for b in bufs])).to(torch.bfloat16)
    assert torch.equal(out16[:count - 1].cpu(), ref16)


def test_dense_average_integers_are_exact(gpu):
    ctx, px, runner = gpu
    rng = np.random.default_rng(22)
    bufs = [inputs.small_integer_values(rng, (10_000,), -100, 100) for _ in range(16)]
    out = torch.empty(10_000, dtype=torch.float32, device="cuda")
    ctx.px_dense_average([runner.to_device(b) for b in bufs], 10_000, out, 1.0 / 16)
    assert np.array_equal(out.cpu().numpy(), oracle.dense_average(bufs))


def test_dense_average_full_size_sampled(gpu):
    """48 x 64M bf16 (the NMT-like dense part) in the benchmark's launch shape (16 launches of 2^22
    output elements, each die working on a contiguous 2^19 of them).  Every worker's buffer is a
    seeded block whose length is odd, rolled by its own shift and repeated, so neither the inputs nor
    the expected output repeat with the launch length or any part of it: a launch, or a die's
    eighth of one, that read or wrote a whole number of its lengths away would be seen.  The oracle
    recomputes windows at both ends, across the borders of launches and of the dies' eighths, and
    a scattered sample."""
    ctx, px, runner = gpu
    w = inputs.NMT
    count = w.dense_count
    launch = 1 << 22
    assert px.px_dense_average_launches(w.n_workers, count, True) == count // launch
    period = launch - 37                                                   # odd: coprime to every power of two
    block = inputs.dense_buffer(w, inputs.dense_rngs(w)[0], period)
    base = runner.to_device(block)
    g = torch.Generator(device="cuda").manual_seed(1808)
    d = []
    for k in range(w.n_workers):                                           # each worker: its own shift
        shift = int(torch.randint(0, period, (1,), generator=g, device="cuda").item())
        d.append(torch.roll(base, shift).repeat(count // period + 1)[:count].contiguous())
    # the expected output at j and at j + launch differ (spot check of the construction itself)
    assert not torch.equal(d[0][:4096], d[0][launch:launch + 4096])
    out = torch.empty(count, dtype=torch.float32, device="cuda")
    ctx.px_dense_average(d, count, out, 1.0 / w.n_workers)
    rng = np.random.default_rng(5)
    picks = [np.arange(0, 4096), np.arange(count // 2 - 777, count // 2 + 777), np.arange(count - 4096, count)]
    for k in (1, 2, 5, 8, 11, 15):                                          # borders between launches
        picks.append(np.arange(k * launch - 1024, k * launch + 1024))
    for k in (1, 3, 9, 20, 63, 127):                                        # borders between the dies' eighths
        picks.append(np.arange(k * (launch >> 3) - 512, k * (launch >> 3) + 512))
    picks.append(np.sort(rng.integers(0, count, size=40_000)))
    for sel in picks:
        t = torch.from_numpy(sel).cuda()
        host = [x[t].view(torch.int16).cpu().numpy().view(np.uint16) for x in d]
        close(out[t].cpu().numpy(), oracle.dense_average(host, average=True))


def test_dense_average_nan_and_inf_with_bf16_output(gpu):
    """A NaN or an infinity in a gradient stays one in the reduced buffer, also when the output is
    rounded to bfloat16 (the rounding bias must not carry a NaN pattern into infinity or zero)."""
    ctx, px, runner = gpu
    count = 4096 + 3
    a = np.zeros(count, dtype=np.float32)
    b = np.ones(count, dtype=np.float32)
    a[5], a[77], a[4097] = np.inf, -np.inf, np.inf
    nan_bits = np.array([0x7F800001, 0xFFFFFFFF, 0x7FC00000, 0xFF80FFFF], dtype=np.uint32).view(np.float32)
    a[100:104] = nan_bits
    a[4098] = nan_bits[0]
    for out_dtype in (torch.bfloat16, torch.float32):
        out = torch.empty(count, dtype=out_dtype, device="cuda")
        ctx.px_dense_average([runner.to_device(a), runner.to_device(b)], count, out, 1.0)
        got = out.float().cpu().numpy()
        ref = oracle.dense_average([a, b], average=False)
        assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.isnan(got).sum() == 5
        assert np.array_equal(np.isinf(got), np.isinf(ref)) and np.array_equal(got[np.isinf(got)], ref[np.isinf(ref)])
        fin = np.isfinite(ref)
        close(got[fin], ref[fin], 1e-2 if out_dtype == torch.bfloat16 else REL_TOL)
    # one buffer, scale 1, bfloat16 output: the library's rounding is the host recipe's, bit for bit
    out = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    ctx.px_dense_average([runner.to_device(a)], count, out, 1.0)
    got_bits = out.view(torch.int16).cpu().numpy().view(np.uint16)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ok = ~np.isnan(a)
    assert np.array_equal(got_bits[ok], want[ok])
    assert np.isnan(inputs.bf16_bits_to_f32(got_bits[~ok])).all()
