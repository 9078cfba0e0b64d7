"""The byte formulas bench.py prices the path with, against the figures they are meant to be.

Algorithmic bytes per call (what the method must move; sort passes and scratch are not credited):
coalesce M*8 + M*D*es + U*8 + U*D*4, partition U*8 + U*4 + (P+1)*8, gradient descent U*(8 + 12*D),
Adagrad U*(8 + 20*D), dense mean N*C*es + C*4.  The expected totals below are those formulas
evaluated by hand for the synthetic workloads (MB = 10^6 bytes), with U counted from the seeded ids.
"""

import numpy as np

import bench
from paper_1808_02621_amd import inputs


def _unique(w, table=0):
    return int(np.unique(np.concatenate(inputs.sparse_ids(w, table))).size)


def test_sparse_bytes_of_the_workloads():
    expected_mb = {            # name: (coalesce, partition, apply), per table, at the measured U
        "tiny": (0.41, 0.006, 0.41),
        "small_lm": (26.7, 0.07, 16.8),
        "large_vocab_lm": (340.9, 0.515, 439.8),
        "nmt_like": (458.6, 0.16, 163.1),
        "stress_zipf": (571.2, 0.6, 128.2),
    }
    for name, (a1, a2, a3) in expected_mb.items():
        w = inputs.WORKLOADS[name]
        u = _unique(w)
        es = 2 if w.val_dtype == "bf16" else 4
        got = bench.sparse_bytes(w.total_rows, u, w.dim, es, w.n_shards, w.optimizer)
        # the formulas, written out once more
        assert got[0] == w.total_rows * 8 + w.total_rows * w.dim * es + u * 8 + u * w.dim * 4
        assert got[1] == u * 8 + u * 4 + (w.n_shards + 1) * 8
        assert got[2] == u * (8 + (12 if w.optimizer == "sgd" else 20) * w.dim)
        for g, e in zip(got, (a1, a2, a3)):
            assert abs(g / 1e6 - e) <= 0.02 * e + 0.005, (name, g / 1e6, e)


def test_dense_bytes_of_the_headline_call():
    w = inputs.NMT
    total = bench.dense_bytes(w.n_workers, w.dense_count, 2)
    assert total == 48 * (1 << 26) * 2 + (1 << 26) * 4 == 6_710_886_400
    assert total // 16 == 419_430_400                      # per launch: 16 launches per call
    lm = inputs.LARGE_LM
    assert bench.dense_bytes(lm.n_workers, lm.dense_count, 4) == 48 * (1 << 23) * 4 + (1 << 23) * 4


def test_measured_statistics_of_the_recipe():
    """Distinct ids per workload: the recipe is seeded, so the counts are exact and any change to it shows here."""
    assert _unique(inputs.TINY) == 526
    assert _unique(inputs.SMALL_LM) == 5_456
    assert _unique(inputs.LARGE_LM) == 42_915
    assert (_unique(inputs.NMT, 0), _unique(inputs.NMT, 1)) == (13_265, 13_323)
    assert _unique(inputs.STRESS_ZIPF) == 49_924
