"""Pins for the oracle's per-worker clipping (Appendix A.3 as printed: each
worker clips its own gradient by its global norm over all layers)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import brute
from oracle import bsgd_oracle as orc


def test_scales_match_numpy_norms_over_tensor_columns_only():
    r = np.random.default_rng(0)
    g = r.standard_normal((6, 50)).astype(np.float32)
    g[:, 20:25] = 1e6                                     # a gap between tensors: must not count
    ranges = [(0, 20), (25, 50)]
    sel = [0, 2, 3, 5]
    norms = [np.linalg.norm(np.concatenate([g[k, 0:20], g[k, 25:50]]).astype(np.float64)) for k in sel]
    c = float(np.median(norms))
    sc = orc.worker_clip_scales(g, sel, ranges, c)
    for s, n in zip(sc, norms):
        assert s == pytest.approx(min(1.0, c / n), rel=1e-14)
    assert (sc < 1).any() and (sc == 1).any()
    for off in (0.0, -1.0, math.inf):
        assert np.array_equal(orc.worker_clip_scales(g, sel, ranges, off), np.ones(4))


def test_step_clips_each_kept_row_then_averages():
    r = np.random.default_rng(1)
    N, b, P = 4, 2, 30
    g = (r.standard_normal((N + b, P)) * r.uniform(0.1, 10, (N + b, 1))).astype(np.float32)
    t = r.random(N + b).astype(np.float32)
    sel, _ = orc.select_first_n(t, N, b)
    th0 = np.zeros(P)
    tz = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    c = 3.0
    orc.step(g, t, N, b, tz, dict(opt="sgd", lr=1.0, worker_clip_norm=c))
    rows = []
    for k in sel:
        row = g[k].astype(np.float64)
        n = np.linalg.norm(row)
        rows.append(row * min(1.0, c / n))
        assert np.linalg.norm(rows[-1]) <= c * (1 + 1e-12)
    np.testing.assert_allclose(tz[0]["theta"], -np.mean(rows, axis=0), rtol=1e-13, atol=1e-16)
    # a huge threshold is the unclipped step
    a = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    u = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    orc.step(g, t, N, b, a, dict(opt="sgd", lr=1.0, worker_clip_norm=1e9))
    orc.step(g, t, N, b, u, dict(opt="sgd", lr=1.0))
    np.testing.assert_array_equal(a[0]["theta"], u[0]["theta"])


def test_dropped_rows_do_not_enter_the_norms():
    r = np.random.default_rng(2)
    N, b, P = 3, 2, 10
    g = r.standard_normal((N + b, P)).astype(np.float32)
    t = np.array([1.0, 5.0, 2.0, 6.0, 3.0], np.float32)
    gn = g.copy()
    gn[[1, 3]] = np.nan
    a = [dict(theta=np.zeros(P), s0=None, s1=None, grad_offset=0)]
    z = [dict(theta=np.zeros(P), s0=None, s1=None, grad_offset=0)]
    orc.step(gn, t, N, b, a, dict(opt="sgd", lr=1.0, worker_clip_norm=0.5))
    g[[1, 3]] = 0
    orc.step(g, t, N, b, z, dict(opt="sgd", lr=1.0, worker_clip_norm=0.5))
    assert np.array_equal(a[0]["theta"], z[0]["theta"]) and np.isfinite(a[0]["theta"]).all()


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("both", [False, True])
def test_brute_force_exact(opt, both):
    r = np.random.default_rng(3)
    N, b, P, T = 3, 1, 5, 3
    hy = dict(opt=opt, lr=0.05, momentum=0.9, decay=0.9, eps=1e-2, worker_clip_norm=1.5,
              clip_norm=0.4 if both else 0.0)
    th0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=np.zeros(P), s1=np.zeros(P), grad_offset=0)]
    theta = [Fraction(float(x)) for x in th0]
    state = dict(v=[Fraction(0)] * P, ms=[Fraction(0)] * P, m=[Fraction(0)] * P)
    for s in range(T):
        g = (r.standard_normal((N + b, P)) * r.uniform(0.2, 3, (N + b, 1))).astype(np.float32)
        t = (1.0 + r.exponential(1.0, N + b)).astype(np.float32)
        kept = brute.ps_collect(t, N, step_tag=s)
        brute.exact_step(g, kept, theta, state, hy)
        ok, sel, _ = orc.step(g, t, N, b, tz, hy)
        assert ok and sorted(kept) == sel.tolist()
    np.testing.assert_allclose(tz[0]["theta"], [float(x) for x in theta], rtol=1e-13, atol=1e-15)
