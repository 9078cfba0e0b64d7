"""Partition-count cost model (Sec. 3.2, Eq. 1): oracle pins, then the library's host functions
against the oracle.  Host arithmetic only; no GPU."""

import math
import os

import numpy as np
import pytest

from oracle import cost_model

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table2_throughput_vs_partitions.txt")


def table2():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        rows[name] = np.array([float(v) for v in vals])
    return np.array([8, 16, 32, 64, 128, 256], dtype=np.float64), rows


# ------------------------------------------------------------------ oracle pins

def test_oracle_fit_recovers_exact_parameters():
    theta = np.array([3.0, 40.0, 0.02])
    p = np.array([2, 4, 8, 16, 32, 64], dtype=np.float64)
    t = theta[0] + theta[1] / p + theta[2] * p                  # Eq. 1 written out
    assert np.allclose(cost_model.fit(p, t), theta, rtol=1e-9)
    # three samples determine the three parameters exactly
    assert np.allclose(cost_model.fit(p[:3], t[:3]), theta, rtol=1e-9)
    # residuals of a least-squares fit are orthogonal to every basis function
    noisy = t + np.array([0.1, -0.2, 0.05, 0.3, -0.1, 0.02])
    th = cost_model.fit(p, noisy)
    res = noisy - cost_model.predict(th, p)
    for basis in (np.ones_like(p), 1 / p, p):
        assert abs(float(res @ basis)) < 1e-8


def test_oracle_minimum_is_sqrt_theta1_over_theta2():
    theta = [1.0, 900.0, 0.25]                                   # critical point sqrt(900 / 0.25) = 60
    best, when = cost_model.argmin(theta, 1, 1000)
    assert best == 60 and math.isclose(when, 1.0 + 15.0 + 15.0)
    assert cost_model.argmin(theta, 1, 32)[0] == 32              # clamped to the sampled range
    assert cost_model.argmin(theta, 100, 400)[0] == 100
    ps = np.arange(1, 500)
    second = np.diff(cost_model.predict(theta, ps), 2)
    assert np.all(second > 0)                                    # convex


def test_oracle_search_order_and_stop():
    curve = {1: 9.0, 2: 6.0, 4: 5.0, 8: 4.0, 16: 3.5, 32: 3.8, 64: 5.0}
    seen = cost_model.search(lambda q: curve[q], 8, 64)
    assert [q for q, _ in seen] == [8, 16, 32, 4]                # up until it rises, then one step down
    seen = cost_model.search(lambda q: curve[q], 32, 64)
    assert [q for q, _ in seen] == [32, 64, 16, 8]
    seen = cost_model.search(lambda q: curve[q], 2, 2)
    assert [q for q, _ in seen] == [2, 1]


def test_oracle_on_the_papers_table_2():
    p, rows = table2()
    # iteration time ~ 1 / throughput; the LM curve falls steeply, flattens, and rises at 256
    t_lm = 1.0 / rows["LM"]
    th = cost_model.fit(p, t_lm)
    assert th[1] > 0 and th[2] > 0                                # both effects of Sec. 3.2 are present
    best, _ = cost_model.argmin(th, 8, 256)
    assert 64 <= best <= 256                                      # inside the sampled range, at its upper end
    assert rows["LM"][4] == rows["LM"].max() and rows["LM"][0] == rows["LM"].min()   # 128 best, 8 worst
    assert math.isclose(rows["LM"].max() / rows["LM"].min(), 1.98, abs_tol=0.03)     # Sec. 2.2 (from unrounded figures)
    assert math.isclose(rows["NMT"].max() / rows["NMT"].min(), 1.12, abs_tol=0.005)
    # starting at the number of machines (8), the sampling rule walks up the LM curve until the first rise (64)
    t_of = dict(zip(p.astype(int).tolist(), t_lm.tolist()))
    t_of[4] = t_of[8] * 1.5                                       # below the table: slower still (Min column, Table 5)
    seen = cost_model.search(lambda q: t_of[q], 8, 256)
    assert [q for q, _ in seen] == [8, 16, 32, 64, 4]


# ------------------------------------------------------- library vs oracle (host)

@pytest.fixture(scope="module")
def px():
    from paper_1808_02621_amd import px as module
    return module


def test_library_fit_and_argmin_match_the_oracle(px):
    rng = np.random.default_rng(0)
    for trial in range(20):
        theta = np.array([rng.uniform(0, 5), rng.uniform(1, 500), rng.uniform(1e-3, 1)])
        p = np.array(sorted(rng.choice(np.arange(1, 300), size=int(rng.integers(3, 9)), replace=False)), dtype=np.float64)
        t = cost_model.predict(theta, p) * (1 + 0.02 * rng.standard_normal(p.size))
        got = px.px_partition_cost_fit(p.tolist(), t.tolist())
        ref = cost_model.fit(p, t)
        assert np.allclose(got, ref, rtol=1e-7, atol=1e-9)
        lo, hi = int(p.min()), int(p.max())
        best, when = px.px_partition_cost_argmin(got, lo, hi)
        o_best, o_when = cost_model.argmin(got, lo, hi)
        assert math.isclose(when, o_when, rel_tol=1e-12) and (best == o_best or math.isclose(
            cost_model.predict(got, best), o_when, rel_tol=1e-12))
    p, rows = table2()
    got = px.px_partition_cost_fit(p.tolist(), (1.0 / rows["NMT"]).tolist())
    assert np.allclose(got, cost_model.fit(p, 1.0 / rows["NMT"]), rtol=1e-7, atol=1e-12)
    with pytest.raises(px.PxError):
        px.px_partition_cost_fit([4, 4, 4], [1, 1, 1])           # one distinct P: singular


@pytest.mark.parametrize("p", [[3, 7, 3, 7], [8, 16, 16, 8, 8], [4, 8, 4], [2, 64, 2], [5, 5, 9, 9, 9, 5]])
def test_library_fit_rejects_two_distinct_partition_counts(px, p):
    """Eq. 1 has three parameters: samples at two partition counts, however often each is repeated,
    do not determine them (the oracle's design matrix has rank 2), and the library must say so
    instead of returning whatever round-off leaves in a singular system."""
    t = [1.0 + 0.37 * i for i in range(len(p))]
    design = np.stack([np.ones(len(p)), 1.0 / np.array(p, dtype=np.float64), np.array(p, dtype=np.float64)], axis=1)
    assert np.linalg.matrix_rank(design) == 2
    with pytest.raises(px.PxError) as err:
        px.px_partition_cost_fit(p, t)
    assert err.value.status == px.PX_ERR_INVALID_ARG
    # a third distinct count makes the same samples acceptable
    got = px.px_partition_cost_fit(p + [11], t + [2.0])
    assert np.allclose(got, cost_model.fit(p + [11], t + [2.0]), rtol=1e-7, atol=1e-9)


def test_library_search_follows_the_same_samples(px):
    rng = np.random.default_rng(1)
    for trial in range(30):
        theta = [rng.uniform(0, 2), rng.uniform(1, 400), rng.uniform(1e-3, 0.5)]
        start = int(2 ** rng.integers(0, 7))
        p_max = int(start * 2 ** rng.integers(0, 6))
        ref = cost_model.search(lambda q: float(cost_model.predict(theta, q)), start, p_max)
        ps, ts = [], []
        while True:
            nxt = px.px_partition_search_next(ps, ts, start, p_max)
            if nxt == 0:
                break
            ps.append(nxt)
            ts.append(float(cost_model.predict(theta, nxt)))
            assert len(ps) <= 64
        assert ps == [q for q, _ in ref]


def test_recorded_search_check_on_flat_noisy_times(px):
    """Times that hardly depend on P (what one GPU measures): the rule still visits the same counts
    as the oracle and the two fits agree, whatever sign the fitted parameters take."""
    import cost_model_checks
    rng = np.random.default_rng(4)
    for trial in range(20):
        start = int(2 ** rng.integers(0, 5))
        p_max = int(start * 2 ** rng.integers(1, 5))
        noise = {}
        ps, ts = [], []
        while True:
            nxt = px.px_partition_search_next(ps, ts, start, p_max)
            if nxt == 0:
                break
            noise.setdefault(nxt, 200.0 + float(rng.normal(0, 1.0)))
            ps.append(nxt)
            ts.append(noise[nxt])
            assert len(ps) <= 32
        cost_model_checks.check_recorded_search(px, cost_model, ps, ts, start, p_max)
