"""Pins for the oracle's arrival-order selection (Algorithm 4, collect loop;
Sec. 3: the first N of N+b gradients are kept, the slowest b dropped).

None of these re-types the oracle's own expression: they use numpy's stable
argsort, an O(W^2) check of the defining property, a message-queue replay of
the collect loop, and hand cases whose answers are evident.
"""
import math

import numpy as np
import pytest

from oracle import brute
from oracle import bsgd_oracle as orc
import workloads as wl


def _defining_property(t, N, sel):
    """|kept| = N and every kept (time, index) key precedes every dropped key."""
    W = len(t)
    kept = set(int(k) for k in sel)
    assert len(kept) == N == len(sel)
    assert list(sel) == sorted(kept)
    for i in kept:
        for j in range(W):
            if j in kept:
                continue
            ti, tj = float(t[i]), float(t[j])
            assert ti < tj or (ti == tj and i < j), (i, j, ti, tj)


@pytest.mark.parametrize("N,b", [(1, 0), (1, 3), (4, 1), (50, 4), (100, 6), (32, 2), (200, 12), (250, 6), (64, 0), (63, 2)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_stable_argsort_and_definition(N, b, seed):
    r = np.random.default_rng(1000 * seed + N + b)
    t = r.lognormal(0.0, 0.4, N + b).astype(np.float32)
    sel, t_step = orc.select_first_n(t, N, b)
    ref = np.sort(np.argsort(t, kind="stable")[:N])
    assert sel.dtype == np.int32
    assert np.array_equal(sel, ref)
    _defining_property(t, N, sel)
    assert t_step == np.sort(t)[N - 1]


@pytest.mark.parametrize("seed", range(20))
def test_ties_go_to_lower_index_like_stable_sort(seed):
    r = np.random.default_rng(seed)
    N, b = 7, 5
    t = r.integers(0, 4, N + b).astype(np.float32)       # many equal times
    sel, t_step = orc.select_first_n(t, N, b)
    assert np.array_equal(sel, np.sort(np.argsort(t, kind="stable")[:N]))
    _defining_property(t, N, sel)


@pytest.mark.parametrize("seed", range(10))
def test_matches_message_queue_replay(seed):
    r = np.random.default_rng(100 + seed)
    N, b = int(r.integers(1, 9)), int(r.integers(0, 4))
    t = (1.0 + r.exponential(1.0, N + b)).astype(np.float32)
    if seed % 2:
        t[r.integers(0, N + b)] = t[0]                    # force a tie
    # the previous step's stragglers show up in the middle of this step and
    # must be dropped by the tag test without displacing anything
    stale = [(float(np.median(t)), int(k)) for k in range(min(b, 2))]
    kept = brute.ps_collect(t, N, step_tag=3, stale=stale)
    sel, t_step = orc.select_first_n(t, N, b)
    assert sorted(kept) == sel.tolist()
    assert float(t[kept[-1]]) == float(t_step)


def test_hand_cases():
    # all equal: the lowest indices win
    sel, ts = orc.select_first_n(np.full(6, 2.5, np.float32), 4, 2)
    assert sel.tolist() == [0, 1, 2, 3] and ts == np.float32(2.5)
    # strictly decreasing: the last N workers are the fastest
    t = np.arange(10, 0, -1).astype(np.float32)
    sel, ts = orc.select_first_n(t, 7, 3)
    assert sel.tolist() == [3, 4, 5, 6, 7, 8, 9] and ts == np.float32(7.0)
    # b = 0: everyone is kept, t_step is the slowest
    t = np.array([3.0, 1.0, 2.0], np.float32)
    sel, ts = orc.select_first_n(t, 3, 0)
    assert sel.tolist() == [0, 1, 2] and ts == np.float32(3.0)
    # N = 1: the single fastest (Algorithm 2's "any worker" is Algorithm 4 with N=1)
    sel, ts = orc.select_first_n(np.array([3.0, 1.0, 2.0], np.float32), 1, 2)
    assert sel.tolist() == [1] and ts == np.float32(1.0)
    # zero of either sign is the same instant
    sel, _ = orc.select_first_n(np.array([0.0, -0.0, 1.0], np.float32), 1, 2)
    assert sel.tolist() == [0]
    sel, _ = orc.select_first_n(np.array([-0.0, 0.0, 1.0], np.float32), 1, 2)
    assert sel.tolist() == [0]
    # negative times order below positive ones
    sel, _ = orc.select_first_n(np.array([0.5, -2.0, -1.0, 3.0], np.float32), 2, 2)
    assert sel.tolist() == [1, 2]


def test_dead_workers():
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    # one dead worker, one backup: the dead one is excluded, step proceeds
    t = np.array([1.0, inf, 2.0, 0.5], np.float32)
    sel, ts = orc.select_first_n(t, 3, 1)
    assert sel.tolist() == [0, 2, 3] and ts == np.float32(2.0)
    # NaN counts as never arriving
    t = np.array([1.0, nan, 2.0, 0.5], np.float32)
    sel, ts = orc.select_first_n(t, 3, 1)
    assert sel.tolist() == [0, 2, 3]
    # b+1 dead workers: the collect loop would wait forever
    t = np.array([1.0, inf, nan, 0.5], np.float32)
    assert orc.select_first_n(t, 3, 1) is None
    assert brute.ps_collect(t, 3) is None
    # -inf is an arrival (the earliest possible)
    t = np.array([1.0, -inf, 2.0], np.float32)
    sel, ts = orc.select_first_n(t, 1, 2)
    assert sel.tolist() == [1]


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        orc.select_first_n(np.zeros(4, np.float32), 4, 1)
    with pytest.raises(ValueError):
        orc.select_first_n(np.zeros(4, np.float32), 0, 4)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_on_workload_arrival_times(name):
    cfg = wl.get_config(name)
    for step in range(cfg.steps):
        t = wl.arrival_times(cfg, step)
        assert t.dtype == np.float32 and t.shape == (cfg.W,)
        sel, t_step = orc.select_first_n(t, cfg.N, cfg.b)
        assert np.array_equal(sel, np.sort(np.argsort(t, kind="stable")[:cfg.N]))
        kept = brute.ps_collect(t, cfg.N)
        assert sorted(kept) == sel.tolist()
        assert math.isfinite(float(t_step))
