"""Benchmark of the sparse/dense gradient aggregation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-others] [--no-cpu] [--separate-streams]

A step is one pass of the whole hot path over one batch of synthetic gradients:
for every sparse variable coalesce -> partition -> apply, then the dense mean.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

The headline workload is the largest configuration (NMT-like: two 32,768 x 1,024
tables with bf16 value rows from 48 workers, plus the mean of 48 bf16 buffers of
64M elements).  The other configurations are timed briefly and reported inside
"other_workloads" (sparse chain and dense mean separately).
"""

from __future__ import annotations

import argparse
import concurrent.futures
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="nmt_like")
    ap.add_argument("--no-others", action="store_true", help="skip the brief runs of the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--separate-streams", action="store_true",
                    help="also time the step with the tables and the dense mean on their own streams (kernels "
                         "then overlap, so leave it out of runs whose per-kernel durations are read)")
    return ap.parse_args()


# -------------------------------------------------------------- byte counting

def sparse_bytes(m, u, dim, es, n_shards, optimizer):
    """Algorithmic HBM bytes of coalesce, partition, apply for one table (unfused)."""
    a1 = m * 8 + m * dim * es + u * 8 + u * dim * 4
    a2 = u * 8 + u * 4 + (n_shards + 1) * 8
    a3 = u * (8 + (12 if optimizer == "sgd" else 20) * dim)
    return a1, a2, a3


def dense_bytes(n, count, es, out_es=4):
    return n * count * es + count * out_es


# ------------------------------------------------------------------ workload

class DeviceWorkload:
    """A workload's inputs in HBM, `sets` rotating copies of the value rows (cold caches)."""

    def __init__(self, w, ctx, sets=1, with_dense=True):
        import torch
        from paper_1808_02621_amd import inputs, px, runner
        self.w, self.ctx, self.runner, self.torch = w, ctx, runner, torch
        hash_code = px.PX_HASH_MUL if w.hash == "mul" else px.PX_HASH_MOD
        self.host_idx, self.host_val, self.tables, self.accums, self.bufs = [], [], [], [], []
        for t in range(w.n_tables):
            idx = inputs.sparse_ids(w, t)
            val = inputs.sparse_values(w, t)
            self.host_idx.append(idx)
            self.host_val.append(val)
            d_idx = [runner.to_device(i) for i in idx]
            per_set = []
            for s in range(sets):
                d_val = [runner.to_device(v) for v in val]
                per_set.append(runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, hash_code))
            self.bufs.append(per_set)
            table = torch.empty((w.vocab, w.dim), dtype=torch.float32, device="cuda")
            table.normal_(0.0, inputs.TABLE_INIT_STD)           # timing only; parity runs use inputs.table_init
            self.tables.append(table)
            self.accums.append(torch.full((w.vocab, w.dim), w.accum_init, dtype=torch.float32, device="cuda")
                               if w.optimizer == "adagrad" else None)
        self.unique = []
        self.dense = []
        self.dense_out = None
        if with_dense and w.dense_count:
            rngs = inputs.dense_rngs(w)
            with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
                host = pool.map(lambda r: inputs.dense_buffer(w, r), rngs)
                for h in host:
                    self.dense.append(runner.to_device(h))
            self.dense_out = torch.empty(w.dense_count, dtype=torch.float32, device="cuda")
        self.step_no = 0

    def sparse(self):
        for t in range(self.w.n_tables):
            b = self.bufs[t][self.step_no % len(self.bufs[t])]
            self.runner.sparse_step(self.ctx, b, self.tables[t], self.accums[t], self.w.optimizer, self.w.lr)

    def sparse_fused(self):
        """The same work through the fused aggregate-and-apply entry points (then partition)."""
        for t in range(self.w.n_tables):
            b = self.bufs[t][self.step_no % len(self.bufs[t])]
            self.runner.fused_step(self.ctx, b, self.tables[t], self.accums[t], self.w.optimizer, self.w.lr)

    def pull_setup(self):
        """The pull side: every worker's ids of every table in one batch, rows gathered in batch order."""
        torch = self.torch
        self.pull_ids = [torch.cat(self.bufs[t][0].idx) for t in range(self.w.n_tables)]
        self.pull_out = torch.empty((self.w.total_rows, self.w.dim), dtype=torch.float32, device="cuda")

    def pull(self):
        for t in range(self.w.n_tables):
            self.ctx.px_sparse_lookup(self.tables[t], self.pull_ids[t], None, self.w.total_rows, None, None,
                                      self.pull_out)

    def pull_bytes(self):
        """Every requested id read and its row written; every distinct row of the table read once."""
        w = self.w
        return sum(w.total_rows * (8 + 4 * w.dim) + u * 4 * w.dim for u in self.unique_counts())

    def dense_mean(self):
        if self.dense:
            self.ctx.px_dense_average(self.dense, self.w.dense_count, self.dense_out, 1.0 / self.w.n_workers)

    def step(self):
        self.sparse()
        self.dense_mean()
        self.step_no += 1

    def overlapped_setup(self):
        """One context and one stream per table, one more pair for the dense mean (a context serves one stream)."""
        from paper_1808_02621_amd import px
        n = self.w.n_tables + (1 if self.dense else 0)
        self.side_ctx = [px.Context(0) for _ in range(n)]
        self.side_streams = [self.torch.cuda.Stream() for _ in range(n)]

    def step_overlapped(self):
        """The same work as step(), the tables and the dense mean side by side on their own streams."""
        torch, w = self.torch, self.w
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)
        for s in self.side_streams:
            s.wait_event(fork)
        if self.dense:
            self.side_ctx[-1].px_dense_average(self.dense, w.dense_count, self.dense_out, 1.0 / w.n_workers,
                                               self.side_streams[-1])
        for t in range(w.n_tables):
            b = self.bufs[t][self.step_no % len(self.bufs[t])]
            self.runner.sparse_step(self.side_ctx[t], b, self.tables[t], self.accums[t], w.optimizer, w.lr,
                                    stream=self.side_streams[t])
        for s in self.side_streams:
            done = torch.cuda.Event()
            done.record(s)
            main.wait_event(done)
        self.step_no += 1

    def unique_counts(self):
        self.torch.cuda.synchronize()
        return [int(self.bufs[t][0].out_num.item()) for t in range(self.w.n_tables)]

    def algorithmic_bytes(self):
        w = self.w
        es = 2 if w.val_dtype == "bf16" else 4
        sp = 0
        for u in self.unique_counts():
            sp += sum(sparse_bytes(w.total_rows, u, w.dim, es, w.n_shards, w.optimizer))
        dn = dense_bytes(w.n_workers, w.dense_count, 2 if w.dense_dtype == "bf16" else 4) if self.dense else 0
        return sp, dn


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.txt" % (kernel, workload))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1]))
    except OSError:
        pass
    return None


def copy_calibration(torch, nbytes=1 << 30, reps=5):
    """A plain device copy of known size: what a streaming kernel reaches on this machine, and the
    reference the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled by."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    pairs = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dst.copy_(src)
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    sec = min(a.elapsed_time(b) for a, b in pairs) * 1e-3
    return {"kernel": "torch copy_, %d MiB read + %d MiB written" % (nbytes >> 20, nbytes >> 20),
            "gbps": 2 * nbytes / sec / 1e9, "frac_of_peak": 2 * nbytes / sec / 1e9 / HBM_PEAK_GBPS}


def event_timed(torch, fn, steps, warmup):
    """Average duration of fn's work on the current stream, from event pairs around each call."""
    for _ in range(warmup):
        fn()
    pairs = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in pairs]
    event_timed.last_median = float(np.median(ms)) * 1e-3
    return float(np.mean(ms)) * 1e-3, float(np.min(ms)) * 1e-3


# --------------------------------------------------------- partition search

def partition_search(torch, px, dw, p_start=8, p_max=256):
    """Sec. 3.2 on this machine: sample the sparse chain's time at the partition counts the paper's
    rule visits (start at 8, the paper's machine count), fit Eq. 1, report the best count in range."""
    saved = [(b.n_shards, b.offsets) for t in dw.bufs for b in t]

    def measure(n_shards):
        for t in dw.bufs:
            for b in t:
                b.n_shards = n_shards
                b.offsets = torch.empty(n_shards + 1, dtype=torch.int64, device="cuda")
        avg, _ = event_timed(torch, dw.sparse, 30, 10)
        return avg * 1e6

    ps, ts = [], []
    while True:
        nxt = px.px_partition_search_next(ps, ts, p_start, p_max)
        if nxt == 0:
            break
        ps.append(nxt)
        ts.append(measure(nxt))
    for extra in (p_start * 2, p_start * 4):            # the fit needs three distinct counts
        if len(ps) < 3 and extra not in ps and extra <= p_max:
            ps.append(extra)
            ts.append(measure(extra))
    out = {"samples_p": ps, "samples_us": ts}
    if len(ps) >= 3:
        theta = px.px_partition_cost_fit(ps, ts)
        best, when = px.px_partition_cost_argmin(theta, min(ps), max(ps))
        out.update({"theta": theta, "best_p": best, "predicted_us": when})
    for (n_shards, offsets), b in zip(saved, [b for t in dw.bufs for b in t]):
        b.n_shards, b.offsets = n_shards, offsets
    return out


# ------------------------------------------------------------ per-call times

def per_call(torch, dw, steps, warmup):
    """Mean duration, achieved GB/s and fraction of peak of each of the three sparse calls
    (all tables of the workload together), from event pairs around each call."""
    w, r = dw.w, dw.runner
    names = ("coalesce", "partition", "apply")
    pairs = {n: [] for n in names}
    for it in range(warmup + steps):
        for t in range(w.n_tables):
            b = dw.bufs[t][dw.step_no % len(dw.bufs[t])]
            calls = (lambda: r.coalesce(dw.ctx, b), lambda: r.partition(dw.ctx, b),
                     lambda: r.apply(dw.ctx, b, dw.tables[t], dw.accums[t], w.optimizer, w.lr))
            for n, call in zip(names, calls):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                call()
                e1.record()
                if it >= warmup:
                    pairs[n].append((t, e0, e1))
        dw.step_no += 1
    torch.cuda.synchronize()
    es = 2 if w.val_dtype == "bf16" else 4
    alg = [0, 0, 0]
    for u in dw.unique_counts():
        for i, x in enumerate(sparse_bytes(w.total_rows, u, w.dim, es, w.n_shards, w.optimizer)):
            alg[i] += x
    out = {}
    for i, n in enumerate(names):
        per_step = sum(e0.elapsed_time(e1) for _, e0, e1 in pairs[n]) * 1e-3 / steps
        out[n] = {"avg_us": per_step * 1e6, "algorithmic_bytes": alg[i], "achieved_gbps": alg[i] / per_step / 1e9,
                  "frac": alg[i] / per_step / 1e9 / HBM_PEAK_GBPS}
    return out


# ------------------------------------------------------- two-level aggregation

def two_level_timing(torch, runner, ctx, b0, w, group, iters=10, warmup=2):
    """Local aggregation per group of `group` workers, then global aggregation of the groups' results
    (Sec. 4.3), against one coalesce of all workers.  Every buffer is allocated before the timed
    regions.  The stages are timed apart, each in a loop of its own so that the device queue stays
    full and an event pair brackets device time only: the group coalesces, the second-level
    coalesce (on the counts read once), the one-level coalesce; the read-back of the groups' counts
    is a synchronisation and is timed with the host clock."""
    t = runner.two_level_buffers(b0.idx, b0.val, w.dim, w.vocab, group)
    runner.two_level_first(ctx, t)
    read_us = []
    for _ in range(iters):
        runner.two_level_first(ctx, t)
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        counts = runner.two_level_read_counts(t)
        read_us.append((time.perf_counter() - h0) * 1e6)
    event_timed(torch, lambda: runner.two_level_first(ctx, t), iters, warmup)
    first = event_timed.last_median
    event_timed(torch, lambda: runner.two_level_second(ctx, t, counts), iters, warmup)
    second = event_timed.last_median
    event_timed(torch, lambda: runner.coalesce(ctx, b0), iters, warmup)
    one = event_timed.last_median
    assert int(t.second.out_num.item()) == int(b0.out_num.item())
    return {
        "what": "coalesce per group of %d workers (%d calls), read the %d counts back, coalesce the groups' results; "
                "all buffers allocated beforehand; medians of %d" % (group, len(t.firsts), len(t.firsts), iters),
        "first_level_us": first * 1e6, "count_readback_us": float(np.median(read_us)), "second_level_us": second * 1e6,
        "two_level_us": first * 1e6 + float(np.median(read_us)) + second * 1e6, "one_level_us": one * 1e6,
        "input_rows": w.total_rows, "rows_into_second_level": int(sum(counts)), "unique_rows": int(b0.out_num.item()),
    }


# ------------------------------------------------------------- sparsity sweep

SWEEP_VOCAB = 50_000
SWEEP_LENGTHS = (120, 60, 30, 15, 8, 4, 1)


def sparsity_sweep(torch, px, ctx, base):
    """The analogue of the paper's Table 6 on this path: the Large-vocab LM recipe at a smaller, fixed
    vocabulary, ids per worker = length x 128 (the paper's batch), one sparse chain timed per length.
    alpha is the fraction of the table's rows a worker's mini-batch touches (Sec. 2.2)."""
    import dataclasses
    from paper_1808_02621_amd import inputs, runner
    out = []
    for length in SWEEP_LENGTHS:
        w = dataclasses.replace(base, name="sparsity_sweep", vocab=SWEEP_VOCAB, n_per_worker=length * 128,
                                n_tables=1, dense_count=0)
        idx = inputs.sparse_ids(w, 0)
        m, u, longest, alpha = inputs.id_statistics(idx, w.vocab)
        d_idx = [runner.to_device(i) for i in idx]
        d_val = [torch.randn((i.numel(), w.dim), dtype=torch.float32, device="cuda") for i in d_idx]   # timing only
        b = runner.sparse_buffers(d_idx, d_val, w.dim, w.vocab, w.n_shards, px.PX_HASH_MUL)
        table = torch.zeros((w.vocab, w.dim), dtype=torch.float32, device="cuda")
        accum = torch.full((w.vocab, w.dim), w.accum_init, dtype=torch.float32, device="cuda")

        def chain(b=b, table=table, accum=accum, w=w):
            runner.sparse_step(ctx, b, table, accum, w.optimizer, w.lr)

        avg, mn = event_timed(torch, chain, 20, 4)
        assert int(b.out_num.item()) == u
        nbytes = sum(sparse_bytes(m, u, w.dim, 4, w.n_shards, w.optimizer))
        out.append({"length": length, "rows_per_worker": length * 128, "input_rows": m, "unique_rows": u,
                    "alpha_worker": alpha, "alpha_all_workers": u / w.vocab, "chain_avg_us": avg * 1e6,
                    "rows_per_s": m / avg, "frac": nbytes / avg / 1e9 / HBM_PEAK_GBPS})
        del b, table, accum, d_val, d_idx
        torch.cuda.empty_cache()
    return {"what": "Large-vocab LM recipe at vocab %d, 48 workers, ids per worker = length x 128" % SWEEP_VOCAB,
            "points": out}


# -------------------------------------------------------------- CPU baseline

def cpu_baseline(dw, sparse_budget_s=5.0, dense_budget_s=5.0):
    """The oracle, as it stands, on one host core: the whole sparse chain of every table, repeated
    until about sparse_budget_s of CPU time is spent, plus the dense mean on a leading slice of
    every buffer sized for about dense_budget_s (scaled up to the whole buffer), as rows per second
    of a step.  Tables are allocated outside the timed region."""
    import oracle
    w = dw.w
    tables = [np.zeros((w.vocab, w.dim), dtype=np.float32) for _ in range(w.n_tables)]
    accums = [np.full((w.vocab, w.dim), w.accum_init, dtype=np.float32) if w.optimizer == "adagrad" else None
              for _ in range(w.n_tables)]
    reps, t_sparse_all = 0, 0.0
    while reps < 1 or (t_sparse_all < sparse_budget_s and reps < 50):
        t0 = time.perf_counter()
        for t in range(w.n_tables):
            ids, rows, _ = oracle.sparse_coalesce(dw.host_idx[t], dw.host_val[t], w.dim, w.vocab)
            _, perm, _ = oracle.partition_rows(ids, w.n_shards, w.hash)
            if w.optimizer == "sgd":
                oracle.sparse_apply_sgd(tables[t], ids, rows, w.lr, perm=perm)
            else:
                oracle.sparse_apply_adagrad(tables[t], accums[t], ids, rows, w.lr, perm=perm)
        t_sparse_all += time.perf_counter() - t0
        reps += 1
    t_sparse = t_sparse_all / reps
    t_dense, dense_note = 0.0, "no dense part"
    if dw.dense:
        def slice_time(n):
            host = [d[:n].view(dw.torch.int16).cpu().numpy().view(np.uint16) if w.dense_dtype == "bf16"
                    else d[:n].cpu().numpy() for d in dw.dense]
            t0 = time.perf_counter()
            oracle.dense_average(host, average=True)
            return time.perf_counter() - t0
        probe_n = max(1, w.dense_count // 64)
        probe = slice_time(probe_n)                               # sizes the real sample
        n = int(min(w.dense_count, max(probe_n, probe_n * dense_budget_s / max(probe, 1e-6))))
        spent = slice_time(n)
        t_dense = spent * w.dense_count / n
        dense_note = "dense mean on the first %d of %d elements of every buffer (%.2f s), scaled to the whole" % (
            n, w.dense_count, spent)
    total = t_sparse + t_dense
    return {
        "value": w.n_tables * w.total_rows / total, "unit": "rows/s", "cores": 1, "kind": "oracle",
        "sample": "full sparse chain of %d table(s), %d repetitions (%.2f s in all, %.3f s each) + %s"
                  % (w.n_tables, reps, t_sparse_all, t_sparse, dense_note),
        "seconds_per_step": total, "host_cpus": os.cpu_count(), "cpu_model": cpu_model(),
    }


def cpu_baseline_all_cores(dw, threads, budget_s=8.0):
    """The same oracle run the way the paper parallelises this work (Sec. 3.2): the incoming indices and
    values of every sparse variable are divided into the P disjoint partitions, and each partition is
    aggregated and applied on its own thread (the shards' rows are disjoint, so the threads share the
    table); the dense mean is split into equal element ranges, one per thread.  The split itself is
    inside the timed region.  The C calls release the interpreter lock."""
    import oracle
    w = dw.w
    pool = concurrent.futures.ThreadPoolExecutor(max_workers=threads)
    tables = [np.zeros((w.vocab, w.dim), dtype=np.float32) for _ in range(w.n_tables)]
    accums = [np.full((w.vocab, w.dim), w.accum_init, dtype=np.float32) if w.optimizer == "adagrad" else None
              for _ in range(w.n_tables)]

    for t in tables:
        t.fill(0.0)                                                # touch the pages outside the timed region

    def one_shard(t, idx_s, val_s):
        ids, rows, _ = oracle.sparse_coalesce([idx_s], [val_s], w.dim, w.vocab)
        if w.optimizer == "sgd":
            oracle.sparse_apply_sgd(tables[t], ids, rows, w.lr)
        else:
            oracle.sparse_apply_adagrad(tables[t], accums[t], ids, rows, w.lr)
        return ids.size

    reps, spent = 0, 0.0
    while reps < 1 or (spent < budget_s / 2 and reps < 50):
        t0 = time.perf_counter()
        jobs = []
        for t in range(w.n_tables):
            ids = np.concatenate(dw.host_idx[t])
            val = np.concatenate(dw.host_val[t])
            shard, _, _ = oracle.partition_rows(ids, w.n_shards, w.hash)      # which partition each incoming row goes to
            for p in range(w.n_shards):
                pick = np.flatnonzero(shard == p)
                jobs.append(pool.submit(one_shard, t, ids[pick], val[pick]))
        uniq = sum(j.result() for j in jobs)
        spent += time.perf_counter() - t0
        reps += 1
    t_sparse = spent / reps
    t_dense, note = 0.0, "no dense part"
    if dw.dense:
        n = int(min(w.dense_count, max(1 << 16, w.dense_count // 8)))
        host = [d[:n].view(dw.torch.int16).cpu().numpy().view(np.uint16) if w.dense_dtype == "bf16"
                else d[:n].cpu().numpy() for d in dw.dense]
        edges = np.linspace(0, n, threads + 1).astype(np.int64)
        t0 = time.perf_counter()
        list(pool.map(lambda k: oracle.dense_average([h[edges[k]:edges[k + 1]] for h in host], average=True),
                      range(threads)))
        spent_d = time.perf_counter() - t0
        t_dense = spent_d * w.dense_count / n
        note = "dense mean on the first %d of %d elements of every buffer in %d ranges (%.2f s), scaled to the whole" % (
            n, w.dense_count, threads, spent_d)
    pool.shutdown()
    total = t_sparse + t_dense
    return {
        "value": w.n_tables * w.total_rows / total, "unit": "rows/s", "cores": threads, "kind": "oracle, one thread per partition",
        "sample": "incoming rows of %d table(s) split into %d partitions, each aggregated and applied on its own thread, "
                  "%d repetitions (%.3f s each, %d distinct rows) + %s" % (w.n_tables, w.n_shards, reps, t_sparse, uniq, note),
        "seconds_per_step": total,
    }


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


# ---------------------------------------------------------------------- main

def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (--gpus %d refused); "
                 "the whole workload runs on cuda:0" % args.gpus)
    import torch
    from paper_1808_02621_amd import inputs, px
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    ctx = px.Context(0)
    w = inputs.WORKLOADS[args.workload]

    calibration = copy_calibration(torch)
    dw = DeviceWorkload(w, ctx, sets=1)
    for _ in range(args.warmup):
        dw.step()
    assert ctx.px_device_status() == px.PX_OK
    uniq = dw.unique_counts()
    sp_bytes, dn_bytes = dw.algorithmic_bytes()

    # the timed region: exactly K steps, with an event pair around the dominant kernel's call
    dense_pairs, step_pairs = [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        s0 = torch.cuda.Event(enable_timing=True)
        s0.record()
        dw.sparse()
        if dw.dense:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            dw.dense_mean()
            b.record()
            dense_pairs.append((a, b))
        s1 = torch.cuda.Event(enable_timing=True)
        s1.record()
        step_pairs.append((s0, s1))
        dw.step_no += 1
    torch.cuda.synchronize()
    sec_per_step = (time.perf_counter() - t0) / args.steps
    step_ms = [a.elapsed_time(b) for a, b in step_pairs]

    rows_per_step = w.n_tables * w.total_rows
    result = {
        "metric": "coalesced+applied gradient rows/sec and achieved HBM GB/s (% of peak), 1 GPU",
        "value": rows_per_step / sec_per_step,
        "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        # the same K steps, each bracketed by an event pair on the stream: median and minimum
        "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(np.min(step_ms)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",      # sums are formed in double; inputs are bf16 or f32, tables and outputs float32
        "data": "synthetic",
        "config": {
            "workload": w.name, "tables": w.n_tables, "vocab": w.vocab, "dim": w.dim,
            "workers": w.n_workers, "rows_per_worker": w.n_per_worker, "zipf_s": w.zipf_s,
            "value_dtype": w.val_dtype, "shards": w.n_shards, "optimizer": w.optimizer,
            "dense_elements": w.dense_count, "dense_dtype": w.dense_dtype, "unique_rows": uniq,
        },
        "step_hbm_gbps": (sp_bytes + dn_bytes) / sec_per_step / 1e9,
        "step_hbm_frac": (sp_bytes + dn_bytes) / sec_per_step / 1e9 / HBM_PEAK_GBPS,
        "step_algorithmic_bytes": {"sparse": sp_bytes, "dense": dn_bytes},
    }

    if dense_pairs:
        ms = [a.elapsed_time(b) for a, b in dense_pairs]
        avg = float(np.mean(ms)) * 1e-3
        # a long output is produced by several launches in a row; the library says how many
        launches = px.px_dense_average_launches(w.n_workers, w.dense_count, w.dense_dtype == "bf16")
        traffic = measured_traffic("k_dense_vec", w.name)
        result["roofline"] = {
            "kernel": "k_dense_vec (px_dense_average, %d launches per call)" % launches, "bound": "hbm",
            "achieved": dn_bytes / avg / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": dn_bytes / avg / 1e9 / HBM_PEAK_GBPS, "traffic": traffic,
            "launches_per_call": launches, "avg_call_us": avg * 1e6,
            "avg_launch_us": avg * 1e6 / launches, "algorithmic_bytes_per_launch": dn_bytes // launches,
        }
    sparse_avg, sparse_min = event_timed(torch, dw.sparse, max(5, args.steps // 2), 2)
    result["sparse_chain"] = {
        "avg_us": sparse_avg * 1e6, "median_us": event_timed.last_median * 1e6, "min_us": sparse_min * 1e6,
        "algorithmic_bytes": sp_bytes,
        "achieved_gbps": sp_bytes / sparse_avg / 1e9, "frac": sp_bytes / sparse_avg / 1e9 / HBM_PEAK_GBPS,
        "rows_per_s": rows_per_step / sparse_avg,
    }

    result["sparse_chain"]["unique_rows_per_s"] = sum(uniq) / sparse_avg
    result["sparse_calls"] = per_call(torch, dw, max(5, args.steps // 2), 2)
    if dw.dense:
        result["roofline"]["elements_per_s"] = w.dense_count / (result["roofline"]["avg_call_us"] * 1e-6)

    fused_avg, fused_min = event_timed(torch, dw.sparse_fused, max(5, args.steps // 2), 2)
    result["sparse_chain_fused"] = {
        "what": "px_sparse_coalesce_apply_* + px_partition_rows: same result, aggregated rows never stored",
        "avg_us": fused_avg * 1e6, "min_us": fused_min * 1e6,
        "achieved_gbps_unfused_bytes": sp_bytes / fused_avg / 1e9,
        "frac_unfused_bytes": sp_bytes / fused_avg / 1e9 / HBM_PEAK_GBPS,
        "rows_per_s": rows_per_step / fused_avg,
    }
    fused_med = event_timed.last_median
    sep_med = result["sparse_chain"]["median_us"] * 1e-6
    result["sparse_chain_best"] = {
        "what": "the faster of the separate calls and the fused entry points on this workload (medians); the fused "
                "path saves 2*U*D*4 bytes and pays unless rows are narrow and heavily duplicated",
        "path": "fused" if fused_med < sep_med else "separate", "median_us": min(fused_med, sep_med) * 1e6,
        "frac_unfused_bytes": sp_bytes / min(fused_med, sep_med) / 1e9 / HBM_PEAK_GBPS,
    }
    # the same step with the independent pieces on their own streams: reported beside the headline,
    # which stays on one stream so that every kernel's duration is its own
    if args.separate_streams:
        dw.overlapped_setup()
        for _ in range(2):
            dw.step_overlapped()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(5, args.steps // 2)):
            dw.step_overlapped()
        torch.cuda.synchronize()
        over = (time.perf_counter() - t0) / max(5, args.steps // 2)
        for c in dw.side_ctx:
            assert c.px_device_status() == px.PX_OK
        result["step_on_separate_streams"] = {
            "what": "the tables' chains and the dense mean enqueued on %d streams (one context each), same results"
                    % len(dw.side_streams),
            "ms_per_step": over * 1e3, "rows_per_s": rows_per_step / over,
            "step_hbm_frac": (sp_bytes + dn_bytes) / over / 1e9 / HBM_PEAK_GBPS,
        }
    dw.pull_setup()
    pull_avg, pull_min = event_timed(torch, dw.pull, max(5, args.steps // 2), 2)
    result["pull_side"] = {
        "what": "px_sparse_lookup: rows of every worker's ids gathered in batch order, all tables; bytes = ids read + "
                "every requested row written + every distinct table row read once",
        "avg_us": pull_avg * 1e6, "algorithmic_bytes": dw.pull_bytes(),
        "achieved_gbps": dw.pull_bytes() / pull_avg / 1e9, "frac": dw.pull_bytes() / pull_avg / 1e9 / HBM_PEAK_GBPS,
    }
    result["copy_calibration"] = calibration
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(dw)
        result["cpu_baseline_all_cores"] = cpu_baseline_all_cores(dw, threads=min(16, os.cpu_count() or 1))
    del dw
    torch.cuda.empty_cache()

    if not args.no_others:
        others = {}
        for name, ow in inputs.WORKLOADS.items():
            if name == w.name:
                continue
            vbytes = ow.total_rows * ow.dim * (2 if ow.val_dtype == "bf16" else 4)
            sets = int(min(4, max(1, (1 << 30) // max(vbytes, 1))))      # > 512 MB of value rows in rotation
            odw = DeviceWorkload(ow, ctx, sets=sets)
            odw.step()
            obytes, odense = odw.algorithmic_bytes()

            def sparse_rot(odw=odw):
                odw.sparse()
                odw.step_no += 1

            def fused_rot(odw=odw):
                odw.sparse_fused()
                odw.step_no += 1

            s_avg, s_min = event_timed(torch, sparse_rot, 20, 4)
            s_med = event_timed.last_median
            f_avg, f_min = event_timed(torch, fused_rot, 20, 4)
            f_med = event_timed.last_median
            entry = {"sparse_median_us": s_med * 1e6, "fused_median_us": f_med * 1e6,
                     "best_path": "fused" if f_med < s_med else "separate",
                     "best_frac_unfused_bytes": obytes / min(f_med, s_med) / 1e9 / HBM_PEAK_GBPS,
                     "input_rows": ow.n_tables * ow.total_rows}
            entry.update({"unique_rows": odw.unique_counts(), "sparse_calls": per_call(torch, odw, 10, 2),
                     "sparse_avg_us": s_avg * 1e6, "sparse_min_us": s_min * 1e6,
                     "sparse_gbps": obytes / s_avg / 1e9, "sparse_frac": obytes / s_avg / 1e9 / HBM_PEAK_GBPS,
                     "rows_per_s": ow.n_tables * ow.total_rows / s_avg,
                     "fused_avg_us": f_avg * 1e6, "fused_frac_unfused_bytes": obytes / f_avg / 1e9 / HBM_PEAK_GBPS})
            if name == "large_vocab_lm":
                entry["partition_search"] = partition_search(torch, px, odw)
                entry["sparsity_sweep"] = sparsity_sweep(torch, px, ctx, ow)
                entry["two_level_aggregation"] = two_level_timing(torch, odw.runner, ctx, odw.bufs[0][0], ow, 6)
            if name == "stress_zipf":
                entry["two_level_aggregation"] = two_level_timing(torch, odw.runner, ctx, odw.bufs[0][0], ow, 8)
            odw.pull_setup()
            p_avg, _ = event_timed(torch, odw.pull, 10, 2)
            entry.update({"pull_avg_us": p_avg * 1e6, "pull_frac": odw.pull_bytes() / p_avg / 1e9 / HBM_PEAK_GBPS})
            if odw.dense:
                d_avg, d_min = event_timed(torch, odw.dense_mean, 10, 2)
                entry.update({"dense_avg_us": d_avg * 1e6, "dense_gbps": odense / d_avg / 1e9,
                              "dense_frac": odense / d_avg / 1e9 / HBM_PEAK_GBPS})
            others[name] = entry
            del odw
            torch.cuda.empty_cache()
        result["other_workloads"] = others

    assert ctx.px_device_status() == px.PX_OK
    print(json.dumps(result))


if __name__ == "__main__":
    main()
