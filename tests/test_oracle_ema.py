"""Pins for the oracle's exponential moving average of the parameters
(Sec. 1.1; last line of Algorithm 4; alpha = 0.9999 in Appendix A)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import brute
from oracle import bsgd_oracle as orc


def test_ema_constant_theta_closed_form():
    th = np.array([1.0, -2.0, 0.5])
    e0 = np.array([0.0, 10.0, 0.5])
    e = e0.copy()
    al, T = 0.9, 25
    for _ in range(T):
        orc.update_ema(e, th, al)
    np.testing.assert_allclose(e, al ** T * e0 + (1 - al ** T) * th, rtol=1e-13)


def test_ema_limits():
    th = np.array([3.0, -1.0])
    e = np.array([7.0, 7.0])
    orc.update_ema(e, th, 1.0)                      # alpha = 1: frozen
    np.testing.assert_array_equal(e, [7.0, 7.0])
    orc.update_ema(e, th, 0.0)                      # alpha = 0: copy of theta(t)
    np.testing.assert_array_equal(e, th)


def test_ema_is_a_geometric_average_of_the_trajectory():
    r = np.random.default_rng(0)
    al, T = 0.7, 9
    traj = r.standard_normal((T, 4))
    e = np.zeros(4)
    for t in range(T):
        orc.update_ema(e, traj[t], al)
    ref = sum((1 - al) * al ** (T - 1 - t) * traj[t] for t in range(T))
    np.testing.assert_allclose(e, ref, rtol=1e-13)


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
def test_step_averages_the_parameters_it_started_from(opt):
    # alpha = 0 makes thetabar(t) a copy of theta(t): after a step it must equal
    # the parameters BEFORE that step's update (the index printed in Algorithm 4)
    r = np.random.default_rng(1)
    N, b, P = 3, 1, 6
    g = r.standard_normal((N + b, P)).astype(np.float32)
    t = r.random(N + b).astype(np.float32)
    th0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=np.zeros(P), s1=np.zeros(P), grad_offset=0, ema=np.full(P, 99.0))]
    hy = dict(opt=opt, lr=0.1, momentum=0.9, decay=0.9, eps=1e-3, clip_norm=0.0, ema_decay=0.0)
    orc.step(g, t, N, b, tz, hy)
    np.testing.assert_array_equal(tz[0]["ema"], th0)
    assert not np.array_equal(tz[0]["theta"], th0)
    th1 = tz[0]["theta"].copy()
    orc.step(g, t, N, b, tz, hy)
    np.testing.assert_array_equal(tz[0]["ema"], th1)


def test_step_without_ema_is_unchanged_and_too_few_freezes_it():
    r = np.random.default_rng(2)
    N, b, P = 3, 1, 5
    g = r.standard_normal((N + b, P)).astype(np.float32)
    t = r.random(N + b).astype(np.float32)
    th0 = r.standard_normal(P)
    a = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    e = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0, ema=th0.copy())]
    hy = dict(opt="sgd", lr=0.1, clip_norm=0.0, ema_decay=0.99)
    orc.step(g, t, N, b, a, hy)
    orc.step(g, t, N, b, e, hy)
    np.testing.assert_array_equal(a[0]["theta"], e[0]["theta"])     # the average does not feed back
    before = e[0]["ema"].copy()
    t_bad = np.array([1.0, np.inf, np.inf, 2.0], np.float32)
    ok, _, _ = orc.step(g, t_bad, N, b, e, hy)
    assert not ok
    np.testing.assert_array_equal(e[0]["ema"], before)


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
def test_brute_force_exact_with_ema(opt):
    r = np.random.default_rng(7)
    N, b, P, T = 3, 2, 4, 4
    hy = dict(opt=opt, lr=0.05, momentum=0.9, decay=0.9, eps=1e-2, clip_norm=0.4, ema_decay=0.9)
    th0 = r.standard_normal(P)
    e0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=np.zeros(P), s1=np.zeros(P), grad_offset=0, ema=e0.copy())]
    theta = [Fraction(float(x)) for x in th0]
    state = dict(v=[Fraction(0)] * P, ms=[Fraction(0)] * P, m=[Fraction(0)] * P, ema=[Fraction(float(x)) for x in e0])
    for s in range(T):
        g = r.standard_normal((N + b, P)).astype(np.float32)
        t = (1.0 + r.exponential(1.0, N + b)).astype(np.float32)
        kept = brute.ps_collect(t, N, step_tag=s)
        brute.exact_step(g, kept, theta, state, hy)
        ok, sel, _ = orc.step(g, t, N, b, tz, hy)
        assert ok and sorted(kept) == sel.tolist()
    np.testing.assert_allclose(tz[0]["ema"], [float(x) for x in state["ema"]], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(tz[0]["theta"], [float(x) for x in theta], rtol=1e-13, atol=1e-15)
