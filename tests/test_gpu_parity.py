"""GPU parity: the HIP library against the CPU oracle on the five workload
configurations, through the C ABI.

Reduced-size cases run the oracle over every element, at sizes that span many
256x4-element chunks and end in a ragged tail.  Full-size cases use the
launch shape the benchmark times; there the oracle follows sampled column
blocks (first, last/ragged, and scattered ones), which is exact because the
un-clipped update is element-wise.  The clipped configuration is checked in
full (its norm couples all elements).
"""
import numpy as np
import pytest

import workloads as wl
from harness import run_parity

pytestmark = pytest.mark.gpu


def _sample_blocks(cfg, k=5, seed=0):
    nb = wl.n_blocks(cfg)
    r = np.random.default_rng(seed)
    mid = r.choice(np.arange(1, nb - 1), size=min(k, nb - 2), replace=False).tolist() if nb > 2 else []
    return sorted(set([0, nb - 1] + [int(x) for x in mid]))


# ---------------------------------------------------------------------------
# reduced sizes, full oracle, every configured step
# ---------------------------------------------------------------------------
def test_c1_full_size_all_elements():
    # C1 is small enough for the oracle as it stands
    res = run_parity(wl.get_config("C1"))
    assert res.P == 1_048_576 and res.steps == 10


def test_c2_reduced_rmsprop_momentum():
    run_parity(wl.scaled_config("C2", 300_007))


def test_c2_reduced_small_eps_exercises_ms():
    # eps = 1.0 swamps ms in the configured workload; eps = 1e-8 makes the
    # running mean square decide the step size
    run_parity(wl.scaled_config("C2", 120_001, eps=1e-8, steps=10))


def test_c3_reduced_momentum_with_warmup():
    run_parity(wl.scaled_config("C3", 200_003))


def test_c4_reduced_multi_tensor_unaligned():
    cfg = wl.scaled_config("C4", 400_000)
    offs, sizes, P = wl.tensor_layout(cfg)
    assert len(sizes) == 300 and any(o % 4 for o in offs)
    run_parity(cfg)


def test_c4_reduced_separate_allocations():
    run_parity(wl.scaled_config("C4", 200_000), steps=4, separate_allocs=True)


def test_c5_reduced_clip_then_momentum():
    P = 64 * 4099
    cfg = wl.scaled_config("C5", P, clip_norm=float(np.sqrt(P / 134_217_728)))
    res = run_parity(cfg)
    assert all(0.3 < s < 0.7 for s in res.clip_scales), res.clip_scales     # clipping is active


# ---------------------------------------------------------------------------
# exponential moving average of theta (last line of Algorithm 4)
# ---------------------------------------------------------------------------
def test_ema_reduced_c2_paper_decay():
    res = run_parity(wl.scaled_config("C2", 150_001), ema_decay=0.9999)
    assert "ema" in res.rel_l2


def test_ema_reduced_c1_sgd_fast_decay():
    run_parity(wl.scaled_config("C1", 70_003), ema_decay=0.5)


def test_ema_reduced_c4_multi_tensor():
    run_parity(wl.scaled_config("C4", 300_000), steps=5, ema_decay=0.9)


def test_ema_reduced_c4_separate_allocations():
    run_parity(wl.scaled_config("C4", 150_000), steps=3, ema_decay=0.99, separate_allocs=True)


def test_ema_reduced_c5_clipped():
    P = 64 * 2051
    cfg = wl.scaled_config("C5", P, clip_norm=float(np.sqrt(P / 134_217_728)))
    run_parity(cfg, ema_decay=0.9)


def test_ema_full_size_c2_sampled():
    cfg = wl.get_config("C2")
    run_parity(cfg, steps=4, sample_blocks=_sample_blocks(cfg, k=3), ema_decay=0.9999)


def test_per_worker_clip_reduced_c2():
    # gradients ~ s_k * N(0,1e-3^2) over P columns: ||G_k|| ~ s_k*1e-3*sqrt(P), s_k in [0.5,1.5]:
    # a threshold at the middle clips about half of the workers
    P = 200_003
    run_parity(wl.scaled_config("C2", P), steps=6, worker_clip=float(1e-3 * np.sqrt(P)))


def test_per_worker_clip_reduced_c4_multi_tensor_and_global_clip():
    cfg = wl.scaled_config("C4", 300_000, clip_norm=2e-4)
    run_parity(cfg, steps=4, worker_clip=1.5)


def test_split_calls_equal_the_step():
    run_parity(wl.scaled_config("C2", 50_001), steps=3, use_split_calls=True)


def test_padded_row_stride():
    run_parity(wl.scaled_config("C3", 70_001), steps=3, ld_extra=64)


# ---------------------------------------------------------------------------
# full sizes, the launch configuration the benchmark uses
# ---------------------------------------------------------------------------
def test_c2_full_size_sampled():
    cfg = wl.get_config("C2")
    res = run_parity(cfg, sample_blocks=_sample_blocks(cfg))
    assert res.P == 25_000_000 and res.steps == 20


def test_c3_full_size_sampled():
    cfg = wl.get_config("C3")
    run_parity(cfg, steps=6, sample_blocks=_sample_blocks(cfg, k=3))     # covers the 5-step warm-up


def test_c4_full_size_sampled():
    cfg = wl.get_config("C4")
    run_parity(cfg, steps=5, sample_blocks=_sample_blocks(cfg, k=6))


def test_c4_full_size_all_elements():
    # every element of the 300-tensor workload under the oracle, so that all of the wide shape's chunks that hold
    # tensor boundaries (about 190 of 2930) are compared, not only those a column sample happens to hit
    cfg = wl.get_config("C4")
    res = run_parity(cfg, steps=2)
    assert res.P == 24_000_429 and res.sampled == 0


def test_c4_full_size_moving_average_sampled():
    cfg = wl.get_config("C4")
    run_parity(cfg, steps=3, sample_blocks=_sample_blocks(cfg, k=8, seed=1), ema_decay=0.9999)


def test_c2_full_size_per_worker_clip_all_elements():
    # each kept gradient clipped by its own norm over all 25 M columns (the per-row sums of squares in the launch
    # shape the benchmark times), then the fused update; the norms couple every element, so the oracle runs in full.
    # ||G_k|| ~ s_k * 1e-3 * sqrt(P) with s_k in [0.5, 1.5]: a threshold at s = 1 clips about half of the workers
    cfg = wl.get_config("C2")
    run_parity(cfg, steps=2, worker_clip=float(1e-3 * np.sqrt(cfg.P)))


def test_c5_full_size_clipped():
    cfg = wl.get_config("C5")
    res = run_parity(cfg, steps=2)
    assert all(0.45 < s < 0.53 for s in res.clip_scales), res.clip_scales
