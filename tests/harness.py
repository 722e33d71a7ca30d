"""Shared driver for the GPU parity tests: runs a workload configuration
through the HIP library and through the CPU oracle on the same fp32 inputs
and applies the three agreement criteria.

  1. the kept worker set (and t_step, status) must match bit-exactly, every step;
  2. theta and each optimizer-state buffer: relative L2 error <= 1e-6 at the end;
  3. per element, |theta_gpu - theta_oracle| <= 8*N*2^-24 * sum over steps and
     kept workers of |g|, checked after 10 steps (or at the end if shorter)
     and at the end.

The oracle keeps theta/state in fp64 across steps; the GPU keeps fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

import workloads as wl
from oracle import bsgd_oracle as orc

REL_L2_TOL = 1e-6
ELEM_FACTOR = 8.0 * 2.0 ** -24


def hyper_dict(cfg, step: int, ema_decay: float = 0.0, worker_clip: float = 0.0) -> Dict:
    """Hyper-parameters as the fp32 values the library receives."""
    f = lambda x: float(np.float32(x))
    return dict(opt=cfg.opt, lr=f(wl.lr_at(cfg, step)), momentum=f(cfg.momentum), decay=f(cfg.decay),
                eps=f(cfg.eps), clip_norm=f(cfg.clip_norm), ema_decay=f(ema_decay), worker_clip_norm=f(worker_clip))


@dataclass
class ParityResult:
    rel_l2: Dict[str, float] = field(default_factory=dict)
    max_bound_ratio: float = 0.0
    steps: int = 0
    P: int = 0
    sampled: int = 0
    clip_scales: List[float] = field(default_factory=list)


def n_state(opt: str) -> int:
    return {"sgd": 0, "momentum": 1, "rmsprop_mom": 2}[opt]


def run_parity(cfg, steps: Optional[int] = None, sample_blocks: Optional[Sequence[int]] = None,
               ld_extra: int = 0, separate_allocs: bool = False, use_split_calls: bool = False,
               ema_decay: Optional[float] = None, worker_clip: float = 0.0, verbose: bool = True) -> ParityResult:
    """sample_blocks: None = oracle over every element; else the oracle only
    follows those column blocks (valid when clipping is off: the update is
    element-wise).  ema_decay: also keep the moving average of theta (started
    at theta0) on both sides and compare it."""
    import torch
    import paper_1604_00981_amd as bs

    steps = cfg.steps if steps is None else steps
    offs, sizes, P = wl.tensor_layout(cfg)
    T = len(sizes)
    W, N, b = cfg.W, cfg.N, cfg.b
    ld = (P + 3) // 4 * 4 + ld_extra
    ns = n_state(cfg.opt)
    clip = cfg.clip_norm > 0
    if sample_blocks is not None and (clip or worker_clip > 0):
        raise ValueError("sampled oracle cannot follow a clipped step")

    dev = "cuda"
    th0 = wl.theta0(cfg)
    # device parameters/state: views into flat buffers (tensor starts then are
    # as unaligned as the packed layout makes them) or separate allocations
    use_ema = ema_decay is not None
    alpha = ema_decay if use_ema else 0.0
    if separate_allocs:
        th_parts = [torch.from_numpy(th0[o:o + n].copy()).to(dev) for o, n in zip(offs, sizes)]
        s_parts = [[torch.zeros(n, device=dev) for n in sizes] for _ in range(ns)]
        e_parts = [t.clone() for t in th_parts] if use_ema else None
    else:
        th_flat = torch.from_numpy(th0).to(dev)
        s_flat = [torch.zeros(P, device=dev) for _ in range(ns)]
        th_parts = [th_flat[o:o + n] for o, n in zip(offs, sizes)]
        s_parts = [[s[o:o + n] for o, n in zip(offs, sizes)] for s in s_flat]
        e_flat = th_flat.clone() if use_ema else None
        e_parts = [e_flat[o:o + n] for o, n in zip(offs, sizes)] if use_ema else None
    items = []
    for j in range(T):
        items.append((th_parts[j], s_parts[0][j] if ns > 0 else None, s_parts[1][j] if ns > 1 else None,
                      offs[j], sizes[j], e_parts[j] if use_ema else None))
    tensors = bs.make_tensors(items)
    hyper0 = bs.make_hyper(**hyper_dict(cfg, 0, alpha, worker_clip))
    ws = bs.alloc_workspace(P, N, b, T, hyper0)
    grads_dev = torch.zeros((W, ld), dtype=torch.float32, device=dev)
    g_pin = torch.zeros((W, ld), dtype=torch.float32, pin_memory=True)   # page-locked staging for uploads
    g_host = g_pin.numpy()
    sel_dev = torch.zeros(N, dtype=torch.int32, device=dev)
    st_dev = torch.zeros(1, dtype=torch.int32, device=dev)
    ts_dev = torch.zeros(1, dtype=torch.float32, device=dev)

    # oracle side
    if sample_blocks is None:
        cols = None
        otz = [dict(theta=th0[o:o + n].astype(np.float64), s0=np.zeros(n) if ns > 0 else None,
                    s1=np.zeros(n) if ns > 1 else None, grad_offset=o,
                    ema=th0[o:o + n].astype(np.float64) if use_ema else None) for o, n in zip(offs, sizes)]
        n_cmp = P
    else:
        cols = wl.block_columns(cfg, sample_blocks)
        n_cmp = cols.shape[0]
        otz = [dict(theta=th0[cols].astype(np.float64), s0=np.zeros(n_cmp) if ns > 0 else None,
                    s1=np.zeros(n_cmp) if ns > 1 else None, grad_offset=0,
                    ema=th0[cols].astype(np.float64) if use_ema else None)]
    abs_sum = np.zeros(n_cmp)
    res = ParityResult(steps=steps, P=P, sampled=0 if cols is None else n_cmp)

    def gpu_theta() -> np.ndarray:
        full = np.concatenate([t.cpu().numpy() for t in th_parts]) if separate_allocs else th_flat.cpu().numpy()
        return full if cols is None else full[cols]

    def gpu_state(i: int) -> np.ndarray:
        full = np.concatenate([t.cpu().numpy() for t in s_parts[i]]) if separate_allocs else s_flat[i].cpu().numpy()
        return full if cols is None else full[cols]

    def gpu_ema() -> np.ndarray:
        full = np.concatenate([t.cpu().numpy() for t in e_parts]) if separate_allocs else e_flat.cpu().numpy()
        return full if cols is None else full[cols]

    def check_bound(tag: str):
        got = gpu_theta().astype(np.float64)
        ref = np.concatenate([t["theta"] for t in otz])
        bound = ELEM_FACTOR * N * abs_sum
        err = np.abs(got - ref)
        ratio = float(np.max(err / np.maximum(bound, 1e-300)))
        res.max_bound_ratio = max(res.max_bound_ratio, ratio)
        assert ratio <= 1.0, f"{cfg.name} {tag}: per-element error is {ratio:.3f}x the bound"

    for step in range(steps):
        wl.grad_matrix(cfg, step, out=g_host, ld=ld)
        t = wl.arrival_times(cfg, step)
        grads_dev.copy_(g_pin)
        t_dev = torch.from_numpy(t).to(dev)
        hy = hyper_dict(cfg, step, alpha, worker_clip)
        hyper = bs.make_hyper(**hy)
        if use_split_calls:
            bs.bsgd_select_first_n(t_dev, N, b, sel_dev, ts_dev, st_dev)
            bs.bsgd_reduce_update(grads_dev, ld, sel_dev, st_dev, N, tensors, hyper, ws)
            torch.cuda.synchronize()
            status, t_step, sel_gpu = int(st_dev.item()), float(ts_dev.item()), sel_dev.cpu().tolist()
        else:
            bs.bsgd_step(grads_dev, ld, t_dev, N, b, tensors, hyper, ws)
            status, t_step = bs.bsgd_last_status(ws)
            sel_gpu = bs.bsgd_last_selection(ws, N)

        if cols is None:
            ogr = g_host
        else:
            ogr = wl.grad_columns(cfg, step, sample_blocks)
            # the generator's block view and the uploaded matrix are the same numbers
            assert np.array_equal(ogr[0], g_host[0, cols])
        ok, sel, ots = orc.step(ogr, t, N, b, otz, hy)
        assert ok and status == 0, (cfg.name, step, status)
        assert sel_gpu == sel.tolist(), f"{cfg.name} step {step}: kept set differs"
        assert np.float32(t_step) == ots, f"{cfg.name} step {step}: t_step differs"
        if clip:
            nrm, sc = bs.bsgd_last_clip(ws)
            res.clip_scales.append(sc)
        for k in sel:
            row = ogr[int(k)]
            abs_sum += np.abs(row[:n_cmp] if cols is not None else row[:P])
        if step + 1 == 10 and steps > 10:
            check_bound("after 10 steps")
        if verbose:
            print(f"  {cfg.name} step {step}: kept set ok, t_step={t_step:.4f}", flush=True)

    check_bound(f"after {steps} steps")
    names = ["theta"] + (["s0"] if ns > 0 else []) + (["s1"] if ns > 1 else []) + (["ema"] if use_ema else [])
    for nm in names:
        got = (gpu_theta() if nm == "theta" else gpu_ema() if nm == "ema"
               else gpu_state(0 if nm == "s0" else 1)).astype(np.float64)
        ref = np.concatenate([t[nm] for t in otz])
        den = np.linalg.norm(ref)
        rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref))
        res.rel_l2[nm] = rel
        assert rel <= REL_L2_TOL, f"{cfg.name}: {nm} relative L2 error {rel:.3e} > {REL_L2_TOL}"
    if verbose:
        print(f"  {cfg.name}: rel L2 {res.rel_l2}, max error/bound {res.max_bound_ratio:.3f}", flush=True)
    return res
