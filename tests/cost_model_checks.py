"""Shared check of a recorded partition-count search (Sec. 3.2, Eq. 1): library against oracle."""

import math

import numpy as np


def check_recorded_search(px, cost_model, ps, ts, start, p_max):
    """ps / ts: the partition counts the library's sampling rule asked for, in order, and the time
    measured at each.  The oracle's search, fed the same times, must ask for the same counts in the
    same order and stop at the same point; both fits and both minimisers must agree."""
    recorded = dict(zip(ps, ts))
    asked = []

    def replay(q):
        assert q in recorded, "the oracle asks for P = %d, which the library never sampled" % q
        asked.append(q)
        return recorded[q]

    ref = cost_model.search(replay, start, p_max)
    assert [q for q, _ in ref] == list(ps)
    assert px.px_partition_search_next(ps, ts, start, p_max) == 0            # and the library agrees it is over
    fit_p, fit_t = list(ps), list(ts)
    if len(set(fit_p)) < 3:
        with np.testing.assert_raises(px.PxError):
            px.px_partition_cost_fit(fit_p, fit_t)
        return None
    got = np.array(px.px_partition_cost_fit(fit_p, fit_t))
    want = cost_model.fit(fit_p, fit_t)
    scale = max(abs(float(v)) for v in fit_t)
    # theta1 and theta2 are scaled by up to max(P) and 1/min(P) against the times
    tol = 1e-7 * scale * np.array([1.0, max(fit_p), 1.0])
    assert np.all(np.abs(got - want) <= tol + 1e-7 * np.abs(want)), (got, want)
    lo, hi = min(fit_p), max(fit_p)
    best, when = px.px_partition_cost_argmin(got.tolist(), lo, hi)
    o_best, o_when = cost_model.argmin(got, lo, hi)
    assert math.isclose(when, o_when, rel_tol=1e-12, abs_tol=1e-12 * scale)
    assert best == o_best or math.isclose(float(cost_model.predict(got, best)), o_when, rel_tol=1e-12)
    return got, best
