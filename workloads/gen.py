"""Deterministic input generators: arrival times, gradient rows, initial
parameters, tensor sizes and the per-step learning rate.

Every random stream is keyed by (seed, step, stream, block), so any block of
any gradient row can be drawn on its own: a test can materialise the whole
(N+b) x P matrix for the device and, separately, only a few column blocks for
a CPU check, and both see the same fp32 values.

Streams: 0 arrival times, 1 straggler mask and factors, 2 per-worker scales,
3 per-tensor scales, 4 tensor sizes, 5 initial parameters, 16+k gradient row
of worker k.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

from .configs import StepConfig

BLOCK = 1 << 16          # elements per independently seeded block of a row

_S_ARRIVAL, _S_STRAGGLER, _S_WSCALE, _S_TSCALE, _S_TSIZE, _S_THETA, _S_ARRIVAL_MANY, _S_ROW0 = 0, 1, 2, 3, 4, 5, 6, 16


def _rng(seed: int, step: int, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, step, stream, block])))


def _threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        n = min(n, int(env))
    return max(1, min(n, 16))


# ----------------------------------------------------------------------------
# arrival times
# ----------------------------------------------------------------------------
def arrival_times(cfg: StepConfig, step: int) -> np.ndarray:
    """fp32[N+b]: when each worker's gradient reaches the parameter side in
    this step.  Drawn in fp64 and cast once; every consumer gets this array."""
    W = cfg.W
    r = _rng(cfg.seed, step, _S_ARRIVAL)
    if cfg.arrival == "shifted_exp":
        t = cfg.arrival_shift + r.exponential(1.0 / cfg.arrival_rate, W)
    elif cfg.arrival == "lognormal":
        t = r.lognormal(0.0, cfg.arrival_sigma, W)
        if cfg.straggler_p > 0.0:
            rs = _rng(cfg.seed, step, _S_STRAGGLER)
            slow = rs.random(W) < cfg.straggler_p
            factor = rs.uniform(cfg.straggler_lo, cfg.straggler_hi, W)
            t = np.where(slow, t * factor, t)
    else:
        raise ValueError(cfg.arrival)
    return t.astype(np.float32)


def arrival_matrix(cfg: StepConfig, iterations: int, workers: Optional[int] = None) -> np.ndarray:
    """fp32[iterations, workers]: arrival times of many recorded iterations at
    once (the raw material of a straggler analysis), from the configuration's
    arrival distribution; a stream of its own, drawn in one go."""
    W = cfg.W if workers is None else int(workers)
    r = _rng(cfg.seed, 0, _S_ARRIVAL_MANY)
    if cfg.arrival == "shifted_exp":
        t = cfg.arrival_shift + r.exponential(1.0 / cfg.arrival_rate, (iterations, W))
    elif cfg.arrival == "lognormal":
        t = r.lognormal(0.0, cfg.arrival_sigma, (iterations, W))
        if cfg.straggler_p > 0.0:
            slow = r.random((iterations, W)) < cfg.straggler_p
            factor = r.uniform(cfg.straggler_lo, cfg.straggler_hi, (iterations, W))
            t = np.where(slow, t * factor, t)
    else:
        raise ValueError(cfg.arrival)
    return t.astype(np.float32)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
def tensor_sizes(cfg: StepConfig) -> List[int]:
    """Element count of each parameter tensor (sums to the real P_total)."""
    if cfg.tensor_mode == "flat":
        return [cfg.P]
    if cfg.tensor_mode == "equal":
        if cfg.P % cfg.T:
            raise ValueError("equal split needs T | P")
        return [cfg.P // cfg.T] * cfg.T
    if cfg.tensor_mode == "loguniform":
        r = _rng(cfg.seed, 0, _S_TSIZE)
        s = np.exp(r.uniform(np.log(cfg.tensor_min), np.log(cfg.tensor_max), cfg.T))
        s = s * (cfg.P / s.sum())
        s = np.maximum(np.rint(s), cfg.tensor_min).astype(np.int64)
        return [int(x) for x in s]        # odd sizes on purpose: unaligned starts
    raise ValueError(cfg.tensor_mode)


def tensor_layout(cfg: StepConfig) -> Tuple[List[int], List[int], int]:
    """(grad_offset per tensor, numel per tensor, P_total): tensors are packed
    back to back inside each gradient row, with no alignment padding."""
    sizes = tensor_sizes(cfg)
    offs, o = [], 0
    for n in sizes:
        offs.append(o)
        o += n
    return offs, sizes, o


def _worker_scales(cfg: StepConfig) -> np.ndarray:
    if cfg.worker_scale is None:
        return np.ones(cfg.W)
    lo, hi = cfg.worker_scale
    return _rng(cfg.seed, 0, _S_WSCALE).uniform(lo, hi, cfg.W)


_scale_cache = {}


def row_scale_vector(cfg: StepConfig) -> Optional[np.ndarray]:
    """fp32[P_total] per-element multiplier carrying the per-tensor scale, or
    None when the configuration has none."""
    if cfg.tensor_scale is None:
        return None
    key = (cfg.name, cfg.seed, cfg.P, cfg.T, cfg.tensor_mode, cfg.tensor_scale, cfg.tensor_max)
    v = _scale_cache.get(key)
    if v is None:
        lo, hi = cfg.tensor_scale
        s = _rng(cfg.seed, 0, _S_TSCALE).uniform(lo, hi, cfg.T).astype(np.float32)
        offs, sizes, total = tensor_layout(cfg)
        v = np.empty(total, dtype=np.float32)
        for o, n, sj in zip(offs, sizes, s):
            v[o:o + n] = sj
        _scale_cache.clear()
        _scale_cache[key] = v
    return v


# ----------------------------------------------------------------------------
# gradients
# ----------------------------------------------------------------------------
def _total(cfg: StepConfig) -> int:
    return tensor_layout(cfg)[2]


def n_blocks(cfg: StepConfig) -> int:
    return (_total(cfg) + BLOCK - 1) // BLOCK


def grad_block(cfg: StepConfig, step: int, row: int, block: int,
               out: Optional[np.ndarray] = None, _ws=None, _tv=None, _P=None) -> np.ndarray:
    """fp32 elements [block*BLOCK, min(P,(block+1)*BLOCK)) of worker `row`'s
    gradient in `step`: sigma * worker_scale * z, then the per-tensor scale."""
    P = _total(cfg) if _P is None else _P
    lo = block * BLOCK
    n = min(BLOCK, P - lo)
    if n <= 0:
        raise IndexError(block)
    ws = _worker_scales(cfg) if _ws is None else _ws
    tv = row_scale_vector(cfg) if _tv is None else _tv
    if out is None:
        out = np.empty(n, dtype=np.float32)
    r = _rng(cfg.seed, step, _S_ROW0 + row, block)
    r.standard_normal(out=out, dtype=np.float32)
    np.multiply(out, np.float32(cfg.grad_sigma * ws[row]), out=out)
    if tv is not None:
        np.multiply(out, tv[lo:lo + n], out=out)
    return out


def grad_row(cfg: StepConfig, step: int, row: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    P = _total(cfg)
    if out is None:
        out = np.empty(P, dtype=np.float32)
    ws, tv = _worker_scales(cfg), row_scale_vector(cfg)
    for blk in range(n_blocks(cfg)):
        lo = blk * BLOCK
        grad_block(cfg, step, row, blk, out=out[lo:min(P, lo + BLOCK)], _ws=ws, _tv=tv, _P=P)
    return out


def grad_matrix(cfg: StepConfig, step: int, out: Optional[np.ndarray] = None,
                ld: Optional[int] = None, threads: Optional[int] = None) -> np.ndarray:
    """fp32[(N+b), ld] (ld >= P_total; columns past P_total are left as they
    are) holding every worker's gradient of this step, row k = worker k."""
    P = _total(cfg)
    ld = P if ld is None else ld
    if out is None:
        out = np.zeros((cfg.W, ld), dtype=np.float32) if ld != P else np.empty((cfg.W, ld), dtype=np.float32)
    ws, tv = _worker_scales(cfg), row_scale_vector(cfg)
    nb = n_blocks(cfg)
    span = 64                                   # blocks per task

    def task(args):
        row, b0 = args
        for blk in range(b0, min(nb, b0 + span)):
            lo = blk * BLOCK
            grad_block(cfg, step, row, blk, out=out[row, lo:min(P, lo + BLOCK)], _ws=ws, _tv=tv, _P=P)

    tasks = [(row, b0) for row in range(cfg.W) for b0 in range(0, nb, span)]
    nthreads = _threads() if threads is None else threads
    if nthreads <= 1 or len(tasks) == 1:
        for t in tasks:
            task(t)
    else:
        with ThreadPoolExecutor(nthreads) as ex:
            list(ex.map(task, tasks))
    return out


def grad_columns(cfg: StepConfig, step: int, blocks: Sequence[int],
                 rows: Optional[Iterable[int]] = None) -> np.ndarray:
    """fp32[(N+b), sum(len(block))]: only the listed column blocks of every
    (or the listed) worker's gradient, concatenated in the order given.  Rows
    not listed are filled with NaN so that reading them cannot go unnoticed."""
    P = _total(cfg)
    lens = [min(BLOCK, P - blk * BLOCK) for blk in blocks]
    out = np.full((cfg.W, int(sum(lens))), np.nan, dtype=np.float32)
    ws, tv = _worker_scales(cfg), row_scale_vector(cfg)
    rows = range(cfg.W) if rows is None else rows
    for row in rows:
        o = 0
        for blk, n in zip(blocks, lens):
            grad_block(cfg, step, row, blk, out=out[row, o:o + n], _ws=ws, _tv=tv, _P=P)
            o += n
    return out


def block_columns(cfg: StepConfig, blocks: Sequence[int]) -> np.ndarray:
    """int64 column indices covered by the listed blocks, in the same order
    as grad_columns lays them out."""
    P = _total(cfg)
    return np.concatenate([np.arange(blk * BLOCK, min(P, (blk + 1) * BLOCK), dtype=np.int64) for blk in blocks])


# ----------------------------------------------------------------------------
# parameters and schedule
# ----------------------------------------------------------------------------
def theta0(cfg: StepConfig) -> np.ndarray:
    """fp32[P_total] initial parameters, N(0, theta_sigma^2), drawn per block."""
    P = _total(cfg)
    out = np.empty(P, dtype=np.float32)
    for blk in range(n_blocks(cfg)):
        lo = blk * BLOCK
        seg = out[lo:min(P, lo + BLOCK)]
        _rng(cfg.seed, 0, _S_THETA, blk).standard_normal(out=seg, dtype=np.float32)
        np.multiply(seg, np.float32(cfg.theta_sigma), out=seg)
    return out


def lr_at(cfg: StepConfig, step: int) -> float:
    """Learning rate handed to the step as gamma_t: constant, or a linear
    warm-up gamma*min(1,(t+1)/warmup)."""
    if cfg.warmup_steps > 0:
        return cfg.lr * min(1.0, (step + 1) / cfg.warmup_steps)
    return cfg.lr
