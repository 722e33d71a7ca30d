#!/usr/bin/env python3
"""Benchmark of the backup-worker Sync-SGD step on one MI355X.

A "step" is one whole pass of the hot path over one batch of synthetic
input: arrival-order selection, gather-sum of the N kept gradient rows,
mean, fused optimizer update.  The workload is configuration C2 (P = 25 M
fp32 parameters in one tensor, N = 50 kept of 54 workers, RMSProp with
momentum), the one the headline metric is quoted on.  Inputs are resident in
HBM before the timed region starts.

Prints ONE JSON line (see the keys below).  `value` is step throughput in
GB/s of algorithmic bytes, (N*P + S*P)*4 per step with S = 6 state streams;
`roofline` prices the dominant kernel alone against the 8 TB/s HBM peak;
`cpu_baseline` times the CPU oracle on a bounded column sample of the same
workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
STATE_STREAMS = {"sgd": 2, "momentum": 4, "rmsprop_mom": 6}


def required_bytes(N: int, P: int, opt: str, ema: bool = False, worker_clip: bool = False) -> int:
    """Algorithmic HBM bytes of one step: N kept rows read once (twice with
    per-worker clipping: norms first), theta and optimizer state (and the
    moving average, if kept) read once and written once."""
    return ((2 if worker_clip else 1) * N * P + (STATE_STREAMS[opt] + (2 if ema else 0)) * P) * 4


def cpu_baseline(cfg, seconds_target: float = 15.0):
    """The oracle as it stands (numpy, fp64, one thread) on a column sample."""
    import numpy as np
    import workloads as wl
    from oracle import bsgd_oracle as orc

    blocks = list(range(32))                                  # 32 x 65536 columns
    n = sum(min(wl.BLOCK, cfg.P - b * wl.BLOCK) for b in blocks)
    g = wl.grad_columns(cfg, 0, blocks)
    hy = dict(opt=cfg.opt, lr=cfg.lr, momentum=cfg.momentum, decay=cfg.decay, eps=cfg.eps, clip_norm=0.0)
    tz = [dict(theta=wl.theta0(cfg)[:n].astype(np.float64), s0=np.zeros(n), s1=np.zeros(n), grad_offset=0)]
    # one untimed step, then as many as fit the target
    orc.step(g, wl.arrival_times(cfg, 0), cfg.N, cfg.b, tz, hy)
    t0 = time.perf_counter()
    reps = 0
    while True:
        orc.step(g, wl.arrival_times(cfg, reps + 1), cfg.N, cfg.b, tz, hy)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= seconds_target or reps >= 400:
            break
    per_step_sample = dt / reps
    gbs = required_bytes(cfg.N, n, cfg.opt) / per_step_sample / 1e9
    full_step_s = per_step_sample * cfg.P / n

    # the same oracle, unchanged, on column slices in a thread pool (numpy releases the GIL inside its loops)
    from concurrent.futures import ThreadPoolExecutor
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    cores = max(1, min(cores, 16))
    cuts = [n * i // cores for i in range(cores + 1)]
    th0 = wl.theta0(cfg)[:n].astype(np.float64)
    parts = [(np.ascontiguousarray(g[:, a:b]),
              [dict(theta=th0[a:b].copy(), s0=np.zeros(b - a), s1=np.zeros(b - a), grad_offset=0)])
             for a, b in zip(cuts[:-1], cuts[1:])]
    with ThreadPoolExecutor(cores) as pool:
        def one(step):
            t = wl.arrival_times(cfg, step)
            list(pool.map(lambda gp: orc.step(gp[0], t, cfg.N, cfg.b, gp[1], hy), parts))
        one(0)
        t0 = time.perf_counter()
        reps_mt = 0
        while True:
            one(reps_mt + 1)
            reps_mt += 1
            dt_mt = time.perf_counter() - t0
            if dt_mt >= seconds_target / 2 or reps_mt >= 400:
                break
    gbs_mt = required_bytes(cfg.N, n, cfg.opt) / (dt_mt / reps_mt) / 1e9
    return {
        "all_cores": {"value": round(gbs_mt, 4), "unit": "GB/s", "cores": cores,
                      "sample": f"{reps_mt} steps, the same columns cut into {cores} slices, one thread each ({dt_mt:.1f} s)"},
        "value": round(gbs, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{reps} steps of the fp64 numpy oracle on the first {n} of {cfg.P} columns, all {cfg.W} rows "
                  f"({dt:.1f} s); scaled to the full width: {full_step_s:.2f} s/step, {1.0 / full_step_s:.3f} steps/s",
        "steps_per_s_full_width": round(1.0 / full_step_s, 4),
    }


def measured_traffic(plain_c2: bool):
    """HBM bytes per launch of the dominant kernel from the committed
    rocprofv3 counter summary (taken on the plain C2 workload), if present."""
    if not plain_c2:
        return None
    p = os.path.join(ROOT, "profiles", "c2_reduce_update_traffic.json")
    try:
        with open(p) as f:
            return json.load(f).get("traffic_bytes_per_launch")
    except (OSError, ValueError):
        return None


def yardstick_main(args, bs) -> int:
    """Plain streaming kernels with the stream mixes of the step's passes (bsgd_yardstick_streams): what the memory
    system gives a kernel that only moves those streams.  One JSON line; every entry is GB/s of bytes moved."""
    import torch
    reps, warm = max(3, args.steps), max(1, args.warmup)

    def run(label, n_floats, n_read, n_write, vec, in_place=True):
        bufs = [torch.full((n_floats,), 0.25, device="cuda") for _ in range(max(n_read, n_write if not in_place else 0))]
        outs = bufs[:n_write] if in_place else [torch.empty(n_floats, device="cuda") for _ in range(n_write)]
        nbytes = n_floats * 4
        for _ in range(warm):
            bs.bsgd_yardstick_streams(bufs[:n_read], outs, nbytes, vec)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            bs.bsgd_yardstick_streams(bufs[:n_read], outs, nbytes, vec)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        moved = (n_read + n_write) * nbytes
        del bufs, outs
        return {"mix": label, "streams_read": n_read, "streams_written": n_write, "MB_per_stream": round(nbytes / 1e6, 1),
                "groups_per_thread": vec, "ms": round(ms, 5), "GB/s": round(moved / (ms * 1e-3) / 1e9, 1),
                "frac_of_peak": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    P2, P5 = 25_000_000, 134_217_728
    rows = []
    for vec in (8, 4, 2, 1):
        rows.append(run("read only, one 5.4 GB buffer (the kept rows of C2)", 54 * P2, 1, 0, vec))
        rows.append(run("update of C2: theta, ms, m read and written in place", P2, 3, 3, vec))
        rows.append(run("pass 2 of a clipped step at C5's size: stored mean, theta, v read; theta, v written", P5, 3, 2, vec))
        rows.append(run("pre-combine of pairs: two rows read, one written", P2, 2, 1, vec, in_place=False))
        rows.append(run("copy: one read, one written", P5, 1, 1, vec, in_place=False))
    print(json.dumps({"metric": "yardstick streaming kernels (bsgd_yardstick_streams)", "unit": "GB/s", "n_gpus": 1,
                      "steps": reps, "warmup": warm, "peak": HBM_PEAK_GBS, "data": "synthetic", "results": rows}))
    return 0


def precombine_main(args, bs, wl) -> int:
    """Times bsgd_precombine on the workload's gradient matrix, machines of G consecutive workers."""
    import numpy as np
    import torch
    cfg = wl.get_config(args.config)
    _, _, P = wl.tensor_layout(cfg)
    W, G = cfg.W, args.precombine
    sizes = [G] * (W // G) + ([W % G] if W % G else [])
    M = len(sizes)
    ld = (P + 3) // 4 * 4
    g_pin = torch.zeros((W, ld), dtype=torch.float32, pin_memory=True)
    wl.grad_matrix(cfg, 0, out=g_pin.numpy(), ld=ld)
    grads = g_pin.cuda()
    del g_pin
    t = torch.from_numpy(wl.arrival_times(cfg, 0)).cuda()
    comb = torch.empty((M, ld), device="cuda")
    when = torch.empty(M, device="cuda")
    cnt = torch.empty(M, dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        bs.bsgd_precombine(grads, ld, P, t, sizes, comb, ld, when, cnt)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        bs.bsgd_precombine(grads, ld, P, t, sizes, comb, ld, when, cnt)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    nbytes = (W + M) * P * 4
    gbs = nbytes / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "pre-combine GB/s (rows read once, machine sums written once)", "value": round(gbs, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: {W} workers on {M} machines of {G}, P={P}"},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}}))
    return 0


def straggler_main(args, bs, wl) -> int:
    """Times bsgd_kth_arrival_times (sorted times and their means) on a recording of B iterations of 100 machines
    with the headline workload's arrival distribution; the oracle is timed beside it on a bounded sample."""
    import numpy as np
    import torch
    from oracle import straggler_oracle as so
    B, W = args.straggler_iterations, 100
    a = wl.arrival_matrix(wl.get_config("C2"), B, workers=W)
    d = torch.from_numpy(a).cuda()
    kth = torch.empty((B, W), device="cuda")
    mean = torch.empty(W, device="cuda", dtype=torch.float64)
    ws = torch.empty(bs.bsgd_straggler_workspace_bytes(W, B), dtype=torch.uint8, device="cuda")
    for _ in range(args.warmup):
        bs.bsgd_kth_arrival_times(d, W, B, kth, mean, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        bs.bsgd_kth_arrival_times(d, W, B, kth, mean, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    nb = min(B, 20000)
    t0 = time.perf_counter()
    ref = so.mean_kth_time(a[:nb])
    cpu_s = time.perf_counter() - t0
    if nb == B:
        assert np.allclose(mean.cpu().numpy(), ref, rtol=1e-12)
    io_bytes = 2 * 4 * B * W                      # every time read once and written once
    slots = 64 * ((W + 63) // 64)
    cmp_rate = B * slots * W / (ms * 1e-3)
    cmp_peak = 256 * 64 * 2.4e9 / 2
    print(json.dumps({
        "metric": "iterations analysed per second (time to collect k gradients, k = 1..100)", "value": round(B / (ms * 1e-3), 1),
        "unit": "iterations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32 keys as u64, f64 sums",
        "data": "synthetic", "config": {"workload": "straggler analysis", "iterations": B, "machines": W},
        "roofline": {"bound": "alu", "achieved": round(cmp_rate / 1e12, 3), "peak": round(cmp_peak / 1e12, 3),
                     "unit": "T key-compares/s", "frac": round(cmp_rate / cmp_peak, 4), "traffic": None,
                     "note": "each of the 64*ceil(W/64) key slots of an iteration is compared with W keys; a compare "
                             "of 64-bit keys plus its count is 2 vector instructions; peak = 256 CUs x 64 lanes x "
                             "2.4 GHz / 2; HBM traffic is only %.0f GB/s" % (io_bytes / (ms * 1e-3) / 1e9)},
        "cpu_baseline": {"value": round(nb / cpu_s, 1), "unit": "iterations/s", "cores": 1, "kind": "oracle",
                         "sample": "first %d iterations" % nb}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C2", help="workload (C2 is the headline; others for exploration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MiB",
                    help="also run plain device copies of this many MiB (yardstick for the profiler's HBM counters)")
    ap.add_argument("--ema-decay", type=float, default=None,
                    help="also keep the moving average of theta (not part of the headline workload)")
    ap.add_argument("--worker-clip", type=float, default=0.0,
                    help="also clip every kept gradient by its own norm (not part of the headline workload)")
    ap.add_argument("--tuning", default="", help="block,vec,unroll,nontemporal override for the reduce kernel")
    ap.add_argument("--ld-pad", type=int, default=0, metavar="ELEMENTS",
                    help="extra elements between gradient rows (exploration: the headline workload has none)")
    ap.add_argument("--precombine", type=int, default=0, metavar="G",
                    help="time bsgd_precombine (one message per machine of G workers) on the workload's gradient "
                         "matrix instead of the step; not the headline workload")
    ap.add_argument("--separate-selection", action="store_true",
                    help="always run the selection as a kernel of its own (small steps otherwise do it inside their "
                         "one launch); for comparison")
    ap.add_argument("--yardstick", action="store_true",
                    help="time plain streaming kernels with the stream mixes of the step's passes instead of the step")
    ap.add_argument("--gap", type=int, default=0, metavar="COLUMNS",
                    help="leave a gap of this many columns in the middle of the gradient rows (a partial-range update: "
                         "the second half of the tensors sits after the gap); exploration, not the headline workload")
    ap.add_argument("--straggler-iterations", type=int, default=0, metavar="B",
                    help="time the straggler analysis (time to collect k gradients over B recorded iterations of "
                         "100 machines) instead of the step; not the headline workload")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step shards along P across GPUs by design, "
              "but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_1604_00981_amd as bs
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.tuning:
        bs.bsgd_set_tuning(*[int(x) for x in args.tuning.split(",")])
    if args.separate_selection:
        bs.bsgd_set_fused_selection(False)

    if args.yardstick:
        return yardstick_main(args, bs)

    if args.straggler_iterations > 0:
        return straggler_main(args, bs, wl)

    if args.precombine > 0:
        return precombine_main(args, bs, wl)

    cfg = wl.get_config(args.config)
    offs, sizes, P = wl.tensor_layout(cfg)
    T, N, b, W = len(sizes), cfg.N, cfg.b, cfg.W
    K, Wm = args.steps, args.warmup
    gap = 4 * max(0, args.gap // 4)
    ld = (P + 3) // 4 * 4 + 4 * max(0, args.ld_pad // 4) + gap
    ns = {"sgd": 0, "momentum": 1, "rmsprop_mom": 2}[cfg.opt]
    # where each tensor's gradient sits in a row: packed, or with the gap before the second half of the tensors
    # (a single tensor is cut in two for that)
    pieces = list(zip(offs, sizes))
    if gap and T == 1:
        half = (P // 2) // 4 * 4
        pieces = [(0, half), (half, P - half)]
    goffs = [o + (gap if gap and j >= len(pieces) // 2 else 0) for j, (o, _) in enumerate(pieces)]

    # ---- inputs, resident in HBM before timing -------------------------------------------
    t_gen = time.perf_counter()
    g_pin = torch.zeros((W, ld), dtype=torch.float32, pin_memory=True)
    wl.grad_matrix(cfg, 0, out=g_pin.numpy(), ld=ld)
    grads = g_pin.cuda()
    del g_pin
    if gap:                                          # move the second half of every row behind the gap, NaN in between
        cut = pieces[len(pieces) // 2][0]
        grads[:, cut + gap:P + gap] = grads[:, cut:P].clone()
        grads[:, cut:cut + gap] = float("nan")
    theta = torch.from_numpy(wl.theta0(cfg)).cuda()
    state = [torch.zeros(P, device="cuda") for _ in range(ns)]
    arrivals = torch.from_numpy(np.stack([wl.arrival_times(cfg, s) for s in range(Wm + 2 * K)])).cuda()
    use_ema = args.ema_decay is not None
    ema = theta.clone() if use_ema else None
    items = [(theta[o:o + n], state[0][o:o + n] if ns > 0 else None, state[1][o:o + n] if ns > 1 else None, go, n,
              ema[o:o + n] if use_ema else None)
             for (o, n), go in zip(pieces, goffs)]
    T = len(items)
    tensors = bs.make_tensors(items)
    hyper = bs.make_hyper(cfg.opt, cfg.lr, cfg.momentum, cfg.decay, cfg.eps, cfg.clip_norm,
                          args.ema_decay if use_ema else 0.0, args.worker_clip)
    ws = bs.alloc_workspace(P + gap, N, b, T, hyper)
    sel = torch.zeros(N, dtype=torch.int32, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t_gen

    stream = torch.cuda.current_stream()
    # what the timed loop hands to the library is prepared before it: one view of the arrival times per step and the
    # stream's handle (small steps are bound by the host's call rate; slicing a tensor costs as much as the call)
    arrival_of = [arrivals[i] for i in range(Wm + 2 * K)]
    handle = stream.cuda_stream

    # ---- warm-up ---------------------------------------------------------------------------
    for i in range(Wm):
        bs.bsgd_step(grads, ld, arrival_of[i], N, b, tensors, hyper, ws, stream=handle)
    torch.cuda.synchronize()

    # ---- timed region: exactly K whole steps -------------------------------------------------
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(K):
        bs.bsgd_step(grads, ld, arrival_of[Wm + i], N, b, tensors, hyper, ws, stream=handle)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / K
    fused_selection = bs.bsgd_last_step_fused_selection()
    status, _ = bs.bsgd_last_status(ws)
    if status != 0:
        print(f"bench.py: step reported status {status}", file=sys.stderr)
        return 1

    # ---- the dominant kernel alone: same steps, events around the reduce/update launch ---------
    ka = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    kb = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    for i in range(K):
        bs.bsgd_select_first_n(arrival_of[Wm + K + i], N, b, sel, None, st, stream=handle)
        ka[i].record(stream)
        bs.bsgd_reduce_update(grads, ld, sel, st, N, tensors, hyper, ws, stream=handle)
        kb[i].record(stream)
    torch.cuda.synchronize()
    launches = max(1, bs.bsgd_last_launch_count())          # the step is cut into launches that each fill the chip once
    kernel_ms_step = sum(a.elapsed_time(c) for a, c in zip(ka, kb)) / K
    kernel_ms = kernel_ms_step / launches                   # average duration of one launch

    if args.calibration_copy > 0:
        nb = args.calibration_copy << 20
        src = torch.ones(nb // 4, device="cuda")
        dst = torch.zeros(nb // 4, device="cuda")
        for _ in range(3):
            bs.bsgd_calibration_copy(dst, src, nb)
        torch.cuda.synchronize()
        del src, dst

    req = required_bytes(N, P, cfg.opt, use_ema, args.worker_clip > 0)
    gbs = req / (ms_per_step * 1e-3) / 1e9
    achieved = (req / launches) / (kernel_ms * 1e-3) / 1e9

    traffic = measured_traffic(cfg.name == "C2" and not use_ema and args.worker_clip <= 0 and not gap
                               and not args.tuning and not args.ld_pad)
    out = {
        "metric": "step GB/s and % of HBM peak at P=25M N=50 b=4 (fused RMSProp); steps/sec",
        "value": round(gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: P={P} fp32 in {T} tensor(s), N={N} kept of {W} workers, {cfg.opt}"
                               + (f", clip {cfg.clip_norm}" if cfg.clip_norm > 0 else "")
                               + (f", moving average alpha={args.ema_decay}" if use_ema else "")
                               + (f", per-worker clip {args.worker_clip}" if args.worker_clip > 0 else "")
                               + (f", a gap of {gap} NaN columns in the middle of every row" if gap else ""),
                   "P": P, "N": N, "b": b, "T": T, "optimizer": cfg.opt, "ld": ld,
                   "required_bytes_per_step": req},
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "steps_per_s": round(1e3 / ms_per_step, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": "profiles/c2_reduce_update_traffic.json (static: rocprofv3 counter runs of this "
                                       "command, not measured in this run)" if traffic is not None else None,
                     "kernel": "k_step (reduce + fused update)", "launches_per_step": launches,
                     "kernel_ms": round(kernel_ms, 5), "kernel_ms_per_step": round(kernel_ms_step, 5),
                     "algorithmic_bytes_per_launch": req // launches},
        "input_setup_s": round(gen_s, 2),
        "selection_inside_the_step_launch": fused_selection,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
