"""CPU oracle for the straggler analysis of Sec. 3.1 of the paper ("Straggler
effects"): how long the parameter side waits for the k-th gradient, and which
split of a fixed pool of N+b machines into N kept workers and b backups is
estimated to converge fastest.

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64; nothing in the product path
may import it, and it imports nothing from the product path.

What Sec. 3.1 computes, in its own order:

  * for every recorded iteration, the time at which the k-th gradient had
    arrived, k = 1..W (the paper plots their distribution and their mean over
    iterations for W = 100 workers);
  * the number of iterations needed to converge when N gradients are
    aggregated, measured for a few N and linearly interpolated in between;
  * their product for every N with N + b = W fixed: the estimated running
    time to convergence; the paper picks the N with the smallest product.

Readings where the paper is silent: a gradient with arrival time +inf or NaN
never arrives (its rank's time is +inf, and so is every mean that contains
it); outside the range of measured N nothing is extrapolated (NaN, never
chosen); among equal smallest products the larger N wins.

Pins (tests/test_oracle_straggler.py): the counting definition of an order
statistic, the message-queue replay of Algorithm 4's collect loop, t_step of
the selection oracle, closed-form means of exponential and uniform order
statistics, the two iteration counts the paper prints and their midpoint, a
hand-worked product table, exact rational replay.  No function here is
unpinned.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def kth_arrival_times(arrival) -> np.ndarray:
    """arrival: [B, W] (or [W]) arrival times of one proxy gradient per worker
    and iteration, as the fp32 values given.  Returns fp32 [B, W]: row i holds
    iteration i's times in the order the parameter side saw them arrive, so
    column k-1 is the time to collect k gradients (Sec. 3.1).  Never-arriving
    gradients (+inf, NaN) come last as +inf."""
    a = np.atleast_2d(np.asarray(arrival, dtype=np.float32))
    a = np.where(np.isnan(a), np.float32(np.inf), a)
    return np.sort(a, axis=1)


def mean_kth_time(arrival) -> np.ndarray:
    """fp64 [W]: mean over iterations of the time to collect k gradients,
    k = 1..W (the curve Sec. 3.1 multiplies with the iteration counts)."""
    kth = kth_arrival_times(arrival).astype(np.float64)
    with np.errstate(invalid="ignore"):
        return kth.sum(axis=0) / kth.shape[0]


def iterations_to_converge(N: float, measured: Sequence[Tuple[float, float]]) -> float:
    """Iterations needed when N gradients are aggregated: the measured points
    (N_i, iterations_i), joined by straight lines (Sec. 3.1).  NaN outside
    the measured range."""
    pts = sorted((float(n), float(it)) for n, it in measured)
    if not pts or N < pts[0][0] or N > pts[-1][0]:
        return float("nan")
    for (n0, i0), (n1, i1) in zip(pts[:-1], pts[1:]):
        if n0 <= N <= n1:
            if n1 == n0:
                return i0
            w = (N - n0) / (n1 - n0)
            return i0 + w * (i1 - i0)
    return pts[-1][1]


def time_to_converge(mean_kth: Sequence[float], measured: Sequence[Tuple[float, float]]):
    """Estimated running time to convergence for every split of W = len(mean_kth)
    machines into N kept and W-N backups: iterations(N) * mean time to collect
    N gradients (Sec. 3.1).  Returns (est fp64[W] indexed by N-1, NaN where
    iterations(N) is unknown; best_N, or 0 if no N has a finite estimate)."""
    W = len(mean_kth)
    est = np.full(W, np.nan)
    for N in range(1, W + 1):
        it = iterations_to_converge(N, measured)
        if it == it:
            est[N - 1] = it * float(mean_kth[N - 1])
    best_N, best = 0, np.inf
    for N in range(1, W + 1):
        e = est[N - 1]
        if np.isfinite(e) and e <= best:
            best, best_N = e, N
    return est, best_N
