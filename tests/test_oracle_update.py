"""Pins for the oracle's reduction, clipping and optimizer updates.

Each check uses a closed form, an invariant, a library routine or exact
arithmetic that does not pass through the oracle's own expressions, chosen so
that a dropped term, a wrong sign, a misplaced learning rate or epsilon, or a
swapped state buffer fails at least one of them.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import bsgd_oracle as orc


# ----------------------------------------------------------------------------
# mean of kept gradients (Algorithm 4, update line; Sec. 1.1 mini-batch mean)
# ----------------------------------------------------------------------------
def test_mean_b0_is_numpy_mean():
    r = np.random.default_rng(0)
    g = r.standard_normal((9, 1000)).astype(np.float32)
    got = orc.reduce_mean(g, list(range(9)))
    assert got.dtype == np.float64
    np.testing.assert_allclose(got, g.astype(np.float64).mean(axis=0), rtol=0, atol=1e-15)


def test_mean_is_exactly_rounded_sum_over_kept_rows_only():
    r = np.random.default_rng(1)
    g = (r.standard_normal((7, 40)) * 10.0 ** r.integers(-6, 6, (7, 40))).astype(np.float32)
    sel = [1, 2, 5, 6]
    got = orc.reduce_mean(g, sel)
    for i in range(g.shape[1]):
        exact = sum(Fraction(float(g[k, i])) for k in sel) / len(sel)
        assert abs(Fraction(float(got[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 49) + Fraction(1, 10 ** 300)
        assert abs(got[i] - math.fsum(float(g[k, i]) for k in sel) / len(sel)) <= 4e-16 * sum(abs(float(g[k, i])) for k in sel)


def test_mean_never_reads_dropped_rows():
    class Guard:
        def __init__(self, g, allowed):
            self.g, self.allowed, self.seen = g, set(allowed), []

        def __getitem__(self, k):
            assert k in self.allowed, f"dropped row {k} was read"
            self.seen.append(k)
            return self.g[k]

    g = np.random.default_rng(2).standard_normal((6, 50)).astype(np.float32)
    guard = Guard(g, [0, 3, 4])
    out = orc.reduce_mean(guard, [0, 3, 4], 10, 30)
    assert sorted(guard.seen) == [0, 3, 4]
    np.testing.assert_allclose(out, g[[0, 3, 4], 10:30].astype(np.float64).mean(axis=0), atol=1e-16)


# ----------------------------------------------------------------------------
# clipping (Appendix A.3: global norm over all layers)
# ----------------------------------------------------------------------------
def test_clip_scale_matches_numpy_norm_over_all_tensors():
    r = np.random.default_rng(3)
    parts = [r.standard_normal(n) for n in (5, 17, 1, 300)]
    nrm = np.linalg.norm(np.concatenate(parts))
    for c in (0.1, 1.0, nrm * 0.999):
        s = orc.clip_scale(parts, c)
        assert s == pytest.approx(c / nrm, rel=1e-14)
        assert np.linalg.norm(np.concatenate([p * s for p in parts])) == pytest.approx(c, rel=1e-13)
    for c in (nrm * (1 + 1e-12), nrm * 1.001, 1e9, math.inf, 0.0, -1.0):
        assert orc.clip_scale(parts, c) == 1.0
    assert orc.clip_scale([np.zeros(4)], 1.0) == 1.0
    # 3-4-5: norm 5 across two tensors, c = 1 -> scale 0.2
    assert orc.clip_scale([np.array([3.0]), np.array([0.0, 4.0])], 1.0) == pytest.approx(0.2, rel=1e-15)


# ----------------------------------------------------------------------------
# SGD (Sec. 1.1)
# ----------------------------------------------------------------------------
def test_sgd_closed_form():
    g = np.array([0.5, -2.0, 0.0, 1e-3])
    th0 = np.array([1.0, 2.0, 3.0, 4.0])
    th = th0.copy()
    lrs = [0.1, 0.2, 0.05, 0.4, 0.01]
    for lr in lrs:
        orc.update_sgd(th, g, lr)
    np.testing.assert_allclose(th, th0 - g * sum(lrs), rtol=1e-15)
    assert th[0] < th0[0] and th[1] > th0[1]            # descent direction


# ----------------------------------------------------------------------------
# momentum SGD
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mu", [0.0, 0.5, 0.9])
def test_momentum_closed_form(mu):
    g = np.array([0.25, -1.5, 3.0])
    th0 = np.array([0.1, 0.2, 0.3])
    th, v = th0.copy(), np.zeros(3)
    lr, T = 0.07, 13
    for t in range(1, T + 1):
        orc.update_momentum(th, v, g, lr, mu)
        v_ref = g * t if mu == 1.0 else g * (1 - mu ** t) / (1 - mu)
        np.testing.assert_allclose(v, v_ref, rtol=1e-13)
    # theta_T = theta_0 - lr * g/(1-mu) * [T - mu (1-mu^T)/(1-mu)]
    ref = th0 - lr * g / (1 - mu) * (T - mu * (1 - mu ** T) / (1 - mu))
    np.testing.assert_allclose(th, ref, rtol=1e-13)


def test_momentum_lr_sits_outside_the_accumulator():
    # with a changing lr the two placements differ; v must not depend on lr
    g = np.array([1.0])
    th, v = np.array([0.0]), np.zeros(1)
    orc.update_momentum(th, v, g, 0.1, 0.5)     # v=1,   th=-0.1
    orc.update_momentum(th, v, g, 1.0, 0.5)     # v=1.5, th=-0.1-1.5
    assert v[0] == pytest.approx(1.5, rel=1e-15)
    assert th[0] == pytest.approx(-1.6, rel=1e-15)


def test_momentum_mu0_is_sgd():
    r = np.random.default_rng(4)
    g, th0 = r.standard_normal(10), r.standard_normal(10)
    a, b, v = th0.copy(), th0.copy(), np.zeros(10)
    orc.update_sgd(a, g, 0.3)
    orc.update_momentum(b, v, g, 0.3, 0.0)
    np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------
# RMSProp with momentum (Appendix A.2/A.3)
# ----------------------------------------------------------------------------
def test_rmsprop_ms_closed_form():
    g = np.array([0.3, -2.0, 1e-4])
    rho = 0.9
    th, ms, m = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 30):
        orc.update_rmsprop_mom(th, ms, m, g, 0.01, 0.9, rho, 1.0)
        np.testing.assert_allclose(ms, g * g * (1 - rho ** t), rtol=1e-12)


def test_rmsprop_sign_sgd_special_case():
    # eps = 0, mu = 0, ms0 = g^2 stays g^2, so each step moves by lr*sign(g):
    # pins the square root and that lr multiplies the normalised gradient
    g = np.array([0.3, -2.0, 1e-4, -7.0])
    th0 = np.array([1.0, 1.0, 1.0, 1.0])
    th, ms, m = th0.copy(), g * g, np.zeros(4)
    lr, T = 0.01, 25
    for _ in range(T):
        orc.update_rmsprop_mom(th, ms, m, g, lr, 0.0, 0.9, 0.0)
    np.testing.assert_allclose(ms, g * g, rtol=1e-12)
    np.testing.assert_allclose(th, th0 - T * lr * np.sign(g), rtol=1e-12)


def test_rmsprop_rho0_is_sign_sgd():
    g = np.array([0.3, -2.0, 5.0])
    th, ms, m = np.zeros(3), np.full(3, 123.0), np.zeros(3)
    orc.update_rmsprop_mom(th, ms, m, g, 0.5, 0.0, 0.0, 0.0)
    np.testing.assert_allclose(th, -0.5 * np.sign(g), rtol=1e-15)


def test_rmsprop_eps_is_inside_the_sqrt():
    # with eps >> ms the step is lr*g/sqrt(eps): eps=4 halves the eps=1 step.
    g = np.array([1e-4, -3e-4])
    outs = []
    for eps in (1.0, 4.0):
        th, ms, m = np.zeros(2), np.zeros(2), np.zeros(2)
        orc.update_rmsprop_mom(th, ms, m, g, 0.045, 0.9, 0.9, eps)
        outs.append(th.copy())
    np.testing.assert_allclose(outs[0], -0.045 * g, rtol=1e-7)
    np.testing.assert_allclose(outs[1], outs[0] / 2.0, rtol=1e-7)
    # eps outside the sqrt would give lr*g/(sqrt(ms)+1) ~ 3e-5 relative off for
    # |g| = 1e-4 * sqrt(0.1); the exact value separates the two readings
    th, ms, m = np.zeros(1), np.zeros(1), np.zeros(1)
    gg = np.array([0.5])
    orc.update_rmsprop_mom(th, ms, m, gg, 1.0, 0.0, 0.0, 1.0)      # ms=0.25
    assert th[0] == pytest.approx(-0.5 / math.sqrt(1.25), rel=1e-15)


def test_rmsprop_momentum_accumulates_scaled_steps():
    # constant g, eps=0, ms0=g^2 (so the normalised gradient is sign(g)):
    # m_t = lr (1-mu^t)/(1-mu) sign(g), theta as for momentum with unit gradient
    g = np.array([2.0, -0.5])
    mu, lr, T = 0.9, 0.02, 17
    th, ms, m = np.zeros(2), g * g, np.zeros(2)
    for t in range(1, T + 1):
        orc.update_rmsprop_mom(th, ms, m, g, lr, mu, 0.5, 0.0)
        np.testing.assert_allclose(m, lr * np.sign(g) * (1 - mu ** t) / (1 - mu), rtol=1e-12)
    ref = -lr * np.sign(g) / (1 - mu) * (T - mu * (1 - mu ** T) / (1 - mu))
    np.testing.assert_allclose(th, ref, rtol=1e-12)


def test_rmsprop_lr_sits_inside_the_accumulator():
    # m keeps steps already scaled by their own lr: changing lr later does not
    # rescale what was accumulated
    g = np.array([1.0])
    th, ms, m = np.zeros(1), np.ones(1), np.zeros(1)
    orc.update_rmsprop_mom(th, ms, m, g, 0.1, 0.5, 1.0, 0.0)   # ms stays 1: m=0.1
    orc.update_rmsprop_mom(th, ms, m, g, 1.0, 0.5, 1.0, 0.0)   # m=0.05+1.0
    assert m[0] == pytest.approx(1.05, rel=1e-15)
    assert th[0] == pytest.approx(-1.15, rel=1e-15)
