"""CPU oracle for one parameter-side step of synchronous SGD with backup
workers (Algorithm 4 of the paper).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 numpy statement of
what the step computes.  It exists so the GPU library can be checked against
something written independently from the paper; nothing in the product path
may import it, and it imports nothing from the product path.

What the step is, in the paper's notation:

  * Algorithm 4, collect loop: the parameter side starts with an empty set,
    waits for gradient messages and keeps those tagged with the current
    step until it holds N of them; with N+b workers sending, the b slowest
    messages are dropped when they arrive (Sec. 3, backup workers).
  * Algorithm 4, update line: theta(t+1) = theta(t) - (gamma_t/N) * sum of the
    kept gradients, i.e. one SGD update (Sec. 1.1) on the mean of the kept
    mini-batch gradients.  Sec. 3 ("Sync-Opt") allows any first-order
    optimizer in place of SGD; Appendix A.2/A.3 name RMSProp with momentum.
  * Appendix A.3: clipping scales the gradient by its global norm taken over
    all layers.
  * Sec. 1.1 and the last line of Algorithm 4: an exponential moving average
    thetabar of the parameters with decay rate alpha (0.9999 in Appendix A).

  * Sec. 6 (work in progress there): gradients of workers that share a
    machine are added on that machine before they are sent; the parameter
    side then receives one message per machine.

Readings where the paper is silent (each is listed in the design notes):
ties in arrival time go to the lower worker index; an arrival time of +inf
or NaN means the message never arrives, and fewer than N arrivals means no
update; momentum is v <- mu v + G, theta <- theta - gamma v; RMSProp with
momentum is ms <- rho ms + (1-rho) G^2, m <- mu m + gamma G / sqrt(ms + eps),
theta <- theta - m; clipping acts on the aggregated mean gradient with
scale min(1, c/||G||); with time-outs in place of backup workers (Sec. 6)
the parameter side listens until the deadline and keeps every current-step
message that came in by then, however many of the N+b that is, and the mean
divides by that number; a machine's combined message leaves when its last
worker is done, N then counts messages, and the mean still divides by the
number of worker gradients the kept messages hold.

Pins (tests/test_oracle_*.py): numpy's stable argsort and an O(W^2)
definition check for the selection, a message-queue simulation of the
collect loop, the plain mean for b=0, exact rational arithmetic on tiny
inputs, NaN-poisoned dropped rows, joint permutation of workers, closed-form
SGD / momentum / RMSProp trajectories for constant gradients, numpy's norm
for clipping, closed forms and exact rational replay for the moving average;
for the time-out variant: the message-queue replay listening until the
deadline, with fewer and with more than N messages in time, a hand case, the
divisor of a whole step, exact replay together with per-worker clipping;
for pre-combined messages: groups of one are the identity, b=0 equals the
plain mean over all workers, uniform groups equal the step on the workers
themselves with their machine's time, exact rational replay.  No function
here is unpinned.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SGD, MOMENTUM, RMSPROP_MOM = "sgd", "momentum", "rmsprop_mom"


# ----------------------------------------------------------------------------
# Algorithm 4, collect loop
# ----------------------------------------------------------------------------
def select_first_n(arrival_t, N: int, b: int):
    """Which N of the N+b gradients the parameter side keeps.

    Algorithm 4 keeps messages in the order they arrive until it has N
    (Sec. 3: "any N workers"; the slowest b are dropped).  Messages are
    ordered by (arrival time, worker index); times are compared as the fp32
    values given.  +inf / NaN = never arrives.

    Returns (sel_idx int32[N] ascending, t_step fp32 = arrival time of the
    N-th kept message) or None when fewer than N messages ever arrive.
    """
    t = np.asarray(arrival_t, dtype=np.float32)
    W = N + b
    if N < 1 or b < 0 or t.shape != (W,):
        raise ValueError("arrival_t must hold N+b times, N >= 1, b >= 0")
    when = [math.inf if math.isnan(float(x)) else float(x) for x in t]
    order = sorted(range(W), key=lambda k: (when[k], k))
    kept = order[:N]
    last = kept[-1]
    if when[last] == math.inf:
        return None
    return np.array(sorted(kept), dtype=np.int32), np.float32(when[last])


def select_ex(arrival_t, N: int, b: int, tags=None, step_tag: int = 0, deadline: float = math.inf,
              n_min: int = 0):
    """Selection with Algorithm 4's tag test spelled out and an optional deadline.

    A message is eligible if its tag equals the current step (Algorithm 4:
    a gradient tagged t' != t is dropped) and it arrives no later than
    `deadline` (Sec. 6 suggests time-outs in place of backup workers).

      n_min == 0  first-N mode: keep the first N eligible messages by
                  (time, index); fewer than N eligible -> None.
      n_min >= 1  deadline mode: keep EVERY eligible message (any number from
                  n_min to N+b); fewer than n_min -> None.  The update then
                  divides by the number kept.

    Returns (sel_idx int32 ascending, t_step fp32 = latest kept arrival) or None.
    """
    t = np.asarray(arrival_t, dtype=np.float32)
    W = N + b
    if N < 1 or b < 0 or t.shape != (W,) or n_min < 0 or n_min > W:
        raise ValueError("bad selection arguments")
    dl = float(np.float32(deadline))
    elig = []
    for k in range(W):
        x = float(t[k])
        if math.isnan(x) or x == math.inf:
            continue                                    # never arrives
        if tags is not None and int(tags[k]) != int(step_tag):
            continue                                    # stale (or foreign) tag: dropped
        if not (x <= dl):
            continue                                    # after the deadline
        elig.append(k)
    order = sorted(elig, key=lambda k: (float(t[k]), k))
    if n_min == 0:
        if len(order) < N:
            return None
        kept = order[:N]
    else:
        if len(order) < n_min:
            return None
        kept = order
    return np.array(sorted(kept), dtype=np.int32), np.float32(t[kept[-1]])


# ----------------------------------------------------------------------------
# Algorithm 4, update line: the mean of the kept gradients
# ----------------------------------------------------------------------------
def reduce_mean(grads, sel_idx: Sequence[int], lo: int = 0, hi: Optional[int] = None) -> np.ndarray:
    """(1/N) * sum over kept workers k of G_k[lo:hi], in fp64.

    `grads` is indexable as grads[k] -> fp32 row of worker k.  Only kept rows
    are touched (dropped gradients play no part in the update)."""
    N = len(sel_idx)
    acc = None
    for k in sel_idx:
        row = np.asarray(grads[int(k)][lo:hi], dtype=np.float64)
        acc = row.copy() if acc is None else acc + row
    return acc / N


def reduce_mean_counted(grads, sel_idx: Sequence[int], row_count: Sequence[int], lo: int = 0,
                        hi: Optional[int] = None) -> np.ndarray:
    """Mean over worker gradients when row k already is the sum of
    row_count[k] of them (Sec. 6): sum of the kept rows / sum of their counts."""
    total = sum(int(row_count[int(k)]) for k in sel_idx)
    acc = None
    for k in sel_idx:
        row = np.asarray(grads[int(k)][lo:hi], dtype=np.float64)
        acc = row.copy() if acc is None else acc + row
    return acc / total


def precombine(grads, arrival_t, group_size: Sequence[int]):
    """Sec. 6: workers that share a machine add their gradients there and
    the machine sends one message.  Workers of machine m are the next
    group_size[m] consecutive rows.  The message leaves when the machine's
    last worker is done (the latest of its workers' times; a worker that
    never finishes holds its machine back for good).

    Returns (combined fp64 [M, width], arrival fp32 [M], row_count int32 [M])."""
    t = np.asarray(arrival_t, dtype=np.float32)
    if sum(int(g) for g in group_size) != t.shape[0] or any(int(g) < 1 for g in group_size):
        raise ValueError("group sizes must be positive and add up to the number of workers")
    rows, when, counts = [], [], []
    k = 0
    for g in group_size:
        g = int(g)
        acc = np.zeros(np.asarray(grads[k]).shape[0], dtype=np.float64)
        latest = -math.inf
        for w in range(k, k + g):
            acc += np.asarray(grads[w], dtype=np.float64)
            x = float(t[w])
            latest = max(latest, math.inf if math.isnan(x) else x)
        rows.append(acc)
        when.append(latest)
        counts.append(g)
        k += g
    return np.stack(rows), np.array(when, dtype=np.float32), np.array(counts, dtype=np.int32)


# ----------------------------------------------------------------------------
# Appendix A.3: clipping by the global norm over all layers
# ----------------------------------------------------------------------------
def clip_scale(gbars: Sequence[np.ndarray], c: float) -> float:
    """min(1, c/||G||) with the 2-norm taken over every tensor together;
    clipping is off for c <= 0 or c = +inf; a zero gradient is left alone."""
    if not (c > 0.0) or math.isinf(c):
        return 1.0
    sq = 0.0
    for g in gbars:
        g = np.asarray(g, dtype=np.float64)
        sq += float(np.dot(g, g))
    nrm = math.sqrt(sq)
    if nrm <= c:
        return 1.0
    return c / nrm


def worker_clip_scales(grads, sel_idx: Sequence[int], ranges: Sequence[Tuple[int, int]], c: float) -> np.ndarray:
    """Appendix A.3 as printed: every worker collects its gradient across all
    layers, computes the global norm ||G_k|| and clips its own gradient.
    Returns, for each kept worker, min(1, c/||G_k||) with the norm taken over
    the columns in `ranges` (the tensors); 1 when c is not positive and finite."""
    out = np.ones(len(sel_idx))
    if not (c > 0.0) or math.isinf(c):
        return out
    for i, k in enumerate(sel_idx):
        sq = 0.0
        for lo, hi in ranges:
            r = np.asarray(grads[int(k)][lo:hi], dtype=np.float64)
            sq += float(np.dot(r, r))
        nrm = math.sqrt(sq)
        if nrm > c:
            out[i] = c / nrm
    return out


def reduce_mean_scaled(grads, sel_idx: Sequence[int], scales: Sequence[float], lo: int, hi: int) -> np.ndarray:
    """(1/N) * sum over kept workers k of scale_k * G_k[lo:hi], in fp64."""
    acc = None
    for k, sc in zip(sel_idx, scales):
        row = np.asarray(grads[int(k)][lo:hi], dtype=np.float64) * float(sc)
        acc = row if acc is None else acc + row
    return acc / len(sel_idx)


# ----------------------------------------------------------------------------
# optimizer updates on the aggregated gradient G (all in place, fp64)
# ----------------------------------------------------------------------------
def update_ema(ema: np.ndarray, theta_before: np.ndarray, alpha: float) -> None:
    """Sec. 1.1 / last line of Algorithm 4: thetabar(t) = alpha thetabar(t-1) +
    (1 - alpha) theta(t), where theta(t) are the parameters step t starts
    from (the printed index: the value before this step's update)."""
    ema *= alpha
    ema += (1.0 - alpha) * theta_before


def update_sgd(theta: np.ndarray, G: np.ndarray, lr: float) -> None:
    """Sec. 1.1: theta(t+1) = theta(t) - gamma_t G(t)."""
    theta -= lr * G


def update_momentum(theta: np.ndarray, v: np.ndarray, G: np.ndarray, lr: float, mu: float) -> None:
    """v <- mu v + G ; theta <- theta - gamma_t v (no dampening, no Nesterov)."""
    v *= mu
    v += G
    theta -= lr * v


def update_rmsprop_mom(theta: np.ndarray, ms: np.ndarray, m: np.ndarray, G: np.ndarray,
                       lr: float, mu: float, rho: float, eps: float) -> None:
    """RMSProp with momentum (Appendix A.2/A.3 give decay rho and momentum
    mu): ms <- rho ms + (1-rho) G^2 ; m <- mu m + gamma_t G/sqrt(ms+eps) ;
    theta <- theta - m."""
    ms *= rho
    ms += (1.0 - rho) * G * G
    m *= mu
    m += lr * G / np.sqrt(ms + eps)
    theta -= m


# ----------------------------------------------------------------------------
# the whole step
# ----------------------------------------------------------------------------
def step(grads, arrival_t, N: int, b: int, tensors: List[Dict], hyper: Dict) -> Tuple[bool, Optional[np.ndarray], Optional[np.float32]]:
    """One parameter-side step.

    grads      indexable by worker k -> fp32 row (length >= every offset+numel)
    arrival_t  fp32[N+b]
    tensors    list of dicts: 'theta' fp64[numel] (updated in place), 's0',
               's1' fp64[numel] or None, 'grad_offset' int, optionally 'ema'
               fp64[numel] (the moving average thetabar, updated in place)
    hyper      dict: opt, lr, momentum, decay, eps, clip_norm, worker_clip_norm,
               ema_decay; and
               optionally tags, step_tag, deadline, n_min (see select_ex);
               optionally row_count int[N+b]: row k is the sum of that many
               worker gradients (see precombine); not together with
               worker_clip_norm

    Returns (ok, sel_idx, t_step).  ok=False (fewer than N arrivals) leaves
    every tensor untouched.
    """
    if any(k in hyper for k in ("tags", "deadline", "n_min")):
        sel = select_ex(arrival_t, N, b, hyper.get("tags"), int(hyper.get("step_tag", 0)),
                        float(hyper.get("deadline", math.inf)), int(hyper.get("n_min", 0)))
    else:
        sel = select_first_n(arrival_t, N, b)
    if sel is None:
        return False, None, None
    sel_idx, t_step = sel

    ranges = [(int(tz["grad_offset"]), int(tz["grad_offset"]) + tz["theta"].shape[0]) for tz in tensors]
    wc = float(hyper.get("worker_clip_norm", 0.0))
    counts = hyper.get("row_count")
    if counts is not None:
        if wc > 0.0 and not math.isinf(wc):
            raise ValueError("a combined message cannot be clipped per worker")
        gbars = [reduce_mean_counted(grads, sel_idx, counts, lo, hi) for lo, hi in ranges]
    elif wc > 0.0 and not math.isinf(wc):               # each worker's own clip comes first
        scales = worker_clip_scales(grads, sel_idx, ranges, wc)
        gbars = [reduce_mean_scaled(grads, sel_idx, scales, lo, hi) for lo, hi in ranges]
    else:
        gbars = [reduce_mean(grads, sel_idx, lo, hi) for lo, hi in ranges]

    s = clip_scale(gbars, float(hyper.get("clip_norm", 0.0)))
    if s != 1.0:
        gbars = [g * s for g in gbars]

    opt = hyper["opt"]
    lr = float(hyper["lr"])
    for tz, G in zip(tensors, gbars):
        if tz.get("ema") is not None:                  # uses theta(t), so it comes before the update
            update_ema(tz["ema"], tz["theta"], float(hyper["ema_decay"]))
        if opt == SGD:
            update_sgd(tz["theta"], G, lr)
        elif opt == MOMENTUM:
            update_momentum(tz["theta"], tz["s0"], G, lr, float(hyper["momentum"]))
        elif opt == RMSPROP_MOM:
            update_rmsprop_mom(tz["theta"], tz["s0"], tz["s1"], G, lr, float(hyper["momentum"]),
                               float(hyper["decay"]), float(hyper["eps"]))
        else:
            raise ValueError(opt)
    return True, sel_idx, t_step
