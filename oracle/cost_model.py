"""Oracle of the partition-count cost model (Parallax Sec. 3.2, Eq. 1).  TEST INFRASTRUCTURE ONLY.

    iter_time(P) = theta0 + theta1 / P + theta2 * P

Plain numpy: a least-squares fit through the library solver, the minimiser by looking at every
integer in the range, and the sampling rule (double from the start until the time goes up, then
halve from the start until it goes up) written as the loop the paper describes.
"""

from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

import numpy as np


def fit(p: Sequence[float], t: Sequence[float]) -> np.ndarray:
    """theta minimising the mean squared error between Eq. 1 and the samples."""
    p = np.asarray(p, dtype=np.float64)
    design = np.stack([np.ones_like(p), 1.0 / p, p], axis=1)
    theta, *_ = np.linalg.lstsq(design, np.asarray(t, dtype=np.float64), rcond=None)
    return theta


def predict(theta: Sequence[float], p) -> np.ndarray:
    p = np.asarray(p, dtype=np.float64)
    return theta[0] + theta[1] / p + theta[2] * p


def argmin(theta: Sequence[float], p_lo: int, p_hi: int) -> Tuple[int, float]:
    """Best integer partition count in [p_lo, p_hi], by exhaustive evaluation."""
    ps = np.arange(p_lo, p_hi + 1)
    times = predict(theta, ps)
    i = int(np.argmin(times))
    return int(ps[i]), float(times[i])


def search(measure: Callable[[int], float], p_start: int, p_max: int) -> List[Tuple[int, float]]:
    """The sampling run of Sec. 3.2; returns the (P, time) pairs in the order they were taken."""
    samples = [(p_start, measure(p_start))]
    prev = samples[0][1]
    q = p_start * 2
    while q <= p_max:
        cur = measure(q)
        samples.append((q, cur))
        if cur > prev:
            break
        prev, q = cur, q * 2
    prev = samples[0][1]
    q = p_start // 2
    while q >= 1:
        cur = measure(q)
        samples.append((q, cur))
        if cur > prev:
            break
        prev, q = cur, q // 2
    return samples
