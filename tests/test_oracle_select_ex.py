"""Pins for the oracle's selection with explicit step tags (Algorithm 4's
`t' == t` test) and with a deadline in place of a fixed count (the time-out
variant the paper's Sec. 6 proposes)."""
import math

import numpy as np
import pytest

from oracle import brute
from oracle import bsgd_oracle as orc


def test_without_options_it_is_the_plain_selection():
    r = np.random.default_rng(0)
    for _ in range(50):
        W = int(r.integers(1, 40))
        N = int(r.integers(1, W + 1))
        t = r.lognormal(0, 0.5, W).astype(np.float32)
        t[r.random(W) < 0.1] = np.inf
        a = orc.select_first_n(t, N, W - N)
        b = orc.select_ex(t, N, W - N)
        assert (a is None) == (b is None)
        if a is not None:
            assert np.array_equal(a[0], b[0]) and a[1] == b[1]


@pytest.mark.parametrize("seed", range(15))
def test_tags_match_the_message_queue_replay(seed):
    r = np.random.default_rng(seed)
    W = int(r.integers(2, 12))
    N = int(r.integers(1, W))
    t = (1.0 + r.exponential(1.0, W)).astype(np.float32)
    tags = np.where(r.random(W) < 0.3, 6, 7).astype(np.int32)      # some messages still carry step 6
    kept = brute.ps_collect(t, N, step_tag=7, tags=tags)
    got = orc.select_ex(t, N, W - N, tags=tags, step_tag=7)
    if kept is None:
        assert got is None
        assert int((tags == 7).sum()) < N
    else:
        assert sorted(kept) == got[0].tolist()
        assert all(tags[k] == 7 for k in kept)
        assert float(t[kept[-1]]) == float(got[1])
        # the same thing as declaring stale messages "never arrived"
        t2 = np.where(tags == 7, t, np.float32(np.inf)).astype(np.float32)
        ref = orc.select_first_n(t2, N, W - N)
        assert np.array_equal(ref[0], got[0])


@pytest.mark.parametrize("seed", range(15))
def test_deadline_keeps_everything_that_came_in_time(seed):
    r = np.random.default_rng(100 + seed)
    W = int(r.integers(2, 14))
    t = (1.0 + r.exponential(1.0, W)).astype(np.float32)
    tags = np.where(r.random(W) < 0.2, 2, 3).astype(np.int32)
    tau = float(np.float32(np.quantile(t, 0.6)))
    n_min = int(r.integers(1, min(4, W) + 1))
    kept = brute.ps_collect(t, n_min, step_tag=3, tags=tags, deadline=tau, keep_all=True)
    got = orc.select_ex(t, W, 0, tags=tags, step_tag=3, deadline=tau, n_min=n_min)
    expect = [k for k in range(W) if tags[k] == 3 and float(t[k]) <= tau]
    if len(expect) < n_min:
        assert got is None and kept is None
    else:
        assert got[0].tolist() == expect == sorted(kept)
        assert float(got[1]) == max(float(t[k]) for k in expect)


def test_hand_cases():
    t = np.array([1.0, 2.0, 3.0, 4.0, 5.0], np.float32)
    # deadline exactly on an arrival: that arrival is in time
    sel, ts = orc.select_ex(t, 5, 0, deadline=3.0, n_min=1)
    assert sel.tolist() == [0, 1, 2] and ts == np.float32(3.0)
    # nobody in time
    assert orc.select_ex(t, 5, 0, deadline=0.5, n_min=1) is None
    # first-N with a deadline: N must be reached by then
    assert orc.select_ex(t, 4, 1, deadline=3.5) is None
    sel, ts = orc.select_ex(t, 3, 2, deadline=3.5)
    assert sel.tolist() == [0, 1, 2]
    # every message stale
    assert orc.select_ex(t, 1, 4, tags=np.zeros(5, np.int32), step_tag=1) is None
    # NaN / inf never arrive, whatever the deadline
    t2 = np.array([np.nan, np.inf, 1.0], np.float32)
    sel, _ = orc.select_ex(t2, 3, 0, deadline=math.inf, n_min=1)
    assert sel.tolist() == [2]


def test_step_divides_by_the_number_kept():
    r = np.random.default_rng(5)
    W, P = 6, 40
    g = r.standard_normal((W, P)).astype(np.float32)
    t = np.array([1.0, 9.0, 2.0, 3.0, 8.0, 2.5], np.float32)
    th0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    ok, sel, ts = orc.step(g, t, W, 0, tz, dict(opt="sgd", lr=0.5, deadline=3.0, n_min=2))
    assert ok and sel.tolist() == [0, 2, 3, 5] and ts == np.float32(3.0)
    ref = th0 - 0.5 * g[[0, 2, 3, 5]].astype(np.float64).mean(axis=0)
    np.testing.assert_allclose(tz[0]["theta"], ref, rtol=1e-14, atol=1e-16)


# ---------------------------------------------------------------------------
# Time-outs in place of backup workers (Sec. 6), with N < N+b: every message
# that is in time is kept, also beyond the N-th; N plays no part in how many.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(20))
def test_deadline_with_backups_keeps_more_than_N_when_more_are_in_time(seed):
    r = np.random.default_rng(300 + seed)
    W = int(r.integers(4, 16))
    N = int(r.integers(1, W - 1))                      # b >= 2
    b = W - N
    t = (1.0 + r.exponential(1.0, W)).astype(np.float32)
    tags = np.where(r.random(W) < 0.15, 8, 9).astype(np.int32)
    tau = float(np.float32(np.quantile(t, r.uniform(0.5, 1.0))))
    n_min = int(r.integers(1, N + 1))
    # the replay listens until the deadline and keeps whatever current-step message came in
    kept = brute.ps_collect(t, n_min, step_tag=9, tags=tags, deadline=tau, keep_all=True)
    got = orc.select_ex(t, N, b, tags=tags, step_tag=9, deadline=tau, n_min=n_min)
    expect = [k for k in range(W) if tags[k] == 9 and float(t[k]) <= tau]
    if len(expect) < n_min:
        assert got is None and kept is None
    else:
        assert got[0].tolist() == expect == sorted(kept)
        assert float(got[1]) == max(float(t[k]) for k in expect)


def test_deadline_with_backups_is_exercised_beyond_N():
    # at least some of the seeded cases above do keep more than N (else they would pin nothing new)
    more = 0
    for seed in range(20):
        r = np.random.default_rng(300 + seed)
        W = int(r.integers(4, 16))
        N = int(r.integers(1, W - 1))
        t = (1.0 + r.exponential(1.0, W)).astype(np.float32)
        tags = np.where(r.random(W) < 0.15, 8, 9).astype(np.int32)
        tau = float(np.float32(np.quantile(t, r.uniform(0.5, 1.0))))
        more += sum(1 for k in range(W) if tags[k] == 9 and float(t[k]) <= tau) > N
    assert more >= 10


def test_deadline_with_backups_hand_case():
    # five workers, N = 2, b = 3; four are in time at tau = 4.5: all four are kept, not the first two
    t = np.array([3.0, 1.0, 5.0, 4.0, 2.0], np.float32)
    sel, ts = orc.select_ex(t, 2, 3, deadline=4.5, n_min=1)
    assert sel.tolist() == [0, 1, 3, 4] and ts == np.float32(4.0)
    # everybody in time: all N+b
    sel, ts = orc.select_ex(t, 2, 3, deadline=5.0, n_min=2)
    assert sel.tolist() == [0, 1, 2, 3, 4] and ts == np.float32(5.0)
    # without the deadline mode (n_min = 0) the same deadline keeps the first N only
    sel, ts = orc.select_ex(t, 2, 3, deadline=4.5, n_min=0)
    assert sel.tolist() == [1, 4] and ts == np.float32(2.0)
    # n_min counts messages in time, whatever N is
    assert orc.select_ex(t, 2, 3, deadline=1.5, n_min=2) is None
    sel, _ = orc.select_ex(t, 2, 3, deadline=1.5, n_min=1)
    assert sel.tolist() == [1]


def test_step_with_backups_divides_by_the_number_kept_not_by_N():
    r = np.random.default_rng(6)
    N, b, P = 2, 4, 30
    g = r.standard_normal((N + b, P)).astype(np.float32)
    t = np.array([1.0, 9.0, 2.0, 3.0, 8.0, 2.5], np.float32)
    th0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=None, s1=None, grad_offset=0)]
    ok, sel, ts = orc.step(g, t, N, b, tz, dict(opt="sgd", lr=0.5, deadline=3.0, n_min=2))
    assert ok and sel.tolist() == [0, 2, 3, 5] and ts == np.float32(3.0)
    ref = th0 - 0.5 * g[[0, 2, 3, 5]].astype(np.float64).sum(axis=0) / 4.0
    np.testing.assert_allclose(tz[0]["theta"], ref, rtol=1e-14, atol=1e-16)
    # and it is not the first-N mean
    first_n = th0 - 0.5 * g[[0, 2]].astype(np.float64).mean(axis=0)
    assert np.abs(tz[0]["theta"] - first_n).max() > 1e-3


def test_step_with_backups_deadline_and_per_worker_clip_exact_replay():
    # the time-out variant together with each worker's own clip (Appendix A.3): the replay keeps what the
    # message queue kept by the deadline and does the arithmetic in rationals
    from fractions import Fraction
    r = np.random.default_rng(7)
    N, b, P = 2, 3, 6
    W = N + b
    g = (r.standard_normal((W, P)) * r.uniform(0.2, 3.0, (W, 1))).astype(np.float32)
    t = np.array([1.5, 1.0, 7.0, 2.0, 1.2], np.float32)
    hy = dict(opt="momentum", lr=0.25, momentum=0.5, worker_clip_norm=2.0, deadline=2.0, n_min=2)
    th0 = r.standard_normal(P)
    tz = [dict(theta=th0.copy(), s0=np.zeros(P), s1=None, grad_offset=0)]
    ok, sel, _ = orc.step(g, t, N, b, tz, hy)
    kept = brute.ps_collect(t, 2, deadline=2.0, keep_all=True)
    assert ok and sorted(kept) == sel.tolist() == [0, 1, 3, 4] and len(kept) > N
    norms = np.linalg.norm(g[sel].astype(np.float64), axis=1)
    assert (norms > 2.0).any() and (norms <= 2.0).any()           # some clipped, some not
    theta = [Fraction(float(x)) for x in th0]
    state = {"v": [Fraction(0)] * P}
    brute.exact_step(g, sorted(kept), theta, state, hy)
    np.testing.assert_allclose(tz[0]["theta"], [float(x) for x in theta], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(tz[0]["s0"], [float(x) for x in state["v"]], rtol=1e-13, atol=1e-15)
