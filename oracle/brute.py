"""Brute-force second implementation used only to pin the oracle on tiny inputs.

TEST INFRASTRUCTURE ONLY.  Nothing here is shared with oracle/bsgd_oracle.py
or with the GPU path.

Two pieces:

  * `ps_collect` plays Algorithm 4's collect loop as a message queue: every
    worker's message (gradient, tag) is delivered at its arrival time, the
    parameter side keeps a message when its tag equals the current step and
    drops it otherwise, and stops listening once it holds N.  Stale messages
    from an earlier step (the previous step's stragglers, Sec. 3) can be
    injected to exercise the tag test.
  * `exact_step` carries out the update line of Algorithm 4 in exact rational
    arithmetic (`fractions.Fraction`); the square root needed by RMSProp
    with momentum is taken with 60-digit `decimal` arithmetic.
"""
from __future__ import annotations

import heapq
import math
from decimal import Decimal, getcontext
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

getcontext().prec = 60


def ps_collect(arrival_t: Sequence[float], N: int, step_tag: int = 0,
               stale: Sequence[Tuple[float, int]] = (), tags: Optional[Sequence[int]] = None,
               deadline: float = math.inf, keep_all: bool = False) -> Optional[List[int]]:
    """Run the collect loop of Algorithm 4 for step `step_tag`.

    arrival_t[k] is when worker k's message tagged `step_tag` is delivered
    (inf/NaN: never).  `stale` lists extra (time, worker) messages carrying
    the tag of the previous step; `tags[k]`, if given, is the tag worker k's
    message carries instead of `step_tag`.  With a finite `deadline` the
    parameter side stops listening at that time; with `keep_all` it keeps
    every current-step message that came in by then (N is then the fewest it
    may proceed with).  Returns the kept workers in the order they were
    kept, or None if the loop would wait forever (or the deadline passes with
    too few).
    """
    queue: List[Tuple[float, int, int, int]] = []   # (time, worker, seq, tag)
    seq = 0
    for k, t in enumerate(arrival_t):
        t = float(t)
        if math.isnan(t) or t == math.inf:
            continue                                # this message is never delivered
        heapq.heappush(queue, (t, k, seq, step_tag if tags is None else int(tags[k])))
        seq += 1
    for t, k in stale:
        heapq.heappush(queue, (float(t), int(k), seq, step_tag - 1))
        seq += 1

    kept: List[int] = []
    while keep_all or len(kept) < N:
        if not queue:
            break                                   # "wait" never returns
        t, k, _, tag = heapq.heappop(queue)
        if t > deadline:
            break                                   # stopped listening
        if tag == step_tag:
            kept.append(k)
        # else: drop the gradient
    if len(kept) < N:
        return None
    return kept


def _sqrt_fraction(x: Fraction) -> Fraction:
    d = (Decimal(x.numerator) / Decimal(x.denominator)).sqrt()
    return Fraction(d)


def exact_step(grads: Sequence[Sequence[float]], kept: Sequence[int], theta: List[Fraction],
               state: Dict[str, List[Fraction]], hyper: Dict) -> None:
    """theta(t+1) from theta(t) and the kept gradients, exactly.  `theta` and
    the lists in `state` ('v' for momentum; 'ms','m' for RMSProp with
    momentum; 'ema' for the moving average of Algorithm 4's last line) are
    updated in place.  Clipping by the global norm of the mean
    gradient is applied when hyper['clip_norm'] is positive and finite."""
    N = len(kept)
    P = len(theta)
    lr = Fraction(hyper["lr"])
    if "ema" in state:                                  # thetabar(t) from theta(t): before the update below
        al = Fraction(hyper["ema_decay"])
        for i in range(P):
            state["ema"][i] = al * state["ema"][i] + (1 - al) * theta[i]
    wc = float(hyper.get("worker_clip_norm", 0.0))
    scale = {k: Fraction(1) for k in kept}
    if wc > 0.0 and not math.isinf(wc):                 # Appendix A.3: each worker clips its own gradient
        for k in kept:
            sq = sum((Fraction(float(grads[k][i])) ** 2 for i in range(P)), Fraction(0))
            if sq > Fraction(wc) * Fraction(wc):
                scale[k] = Fraction(wc) / _sqrt_fraction(sq)
    G = []
    for i in range(P):
        s = Fraction(0)
        for k in kept:
            s += scale[k] * Fraction(float(grads[k][i]))
        G.append(s / N)

    c = float(hyper.get("clip_norm", 0.0))
    if c > 0.0 and not math.isinf(c):
        sq = sum((g * g for g in G), Fraction(0))
        if sq > Fraction(c) * Fraction(c):
            scale = Fraction(c) / _sqrt_fraction(sq)
            G = [g * scale for g in G]

    opt = hyper["opt"]
    if opt == "sgd":
        for i in range(P):
            theta[i] -= lr * G[i]
    elif opt == "momentum":
        mu = Fraction(hyper["momentum"])
        v = state["v"]
        for i in range(P):
            v[i] = mu * v[i] + G[i]
            theta[i] -= lr * v[i]
    elif opt == "rmsprop_mom":
        mu, rho, eps = Fraction(hyper["momentum"]), Fraction(hyper["decay"]), Fraction(hyper["eps"])
        ms, m = state["ms"], state["m"]
        for i in range(P):
            ms[i] = rho * ms[i] + (1 - rho) * G[i] * G[i]
            m[i] = mu * m[i] + lr * G[i] / _sqrt_fraction(ms[i] + eps)
            theta[i] -= m[i]
    else:
        raise ValueError(opt)
