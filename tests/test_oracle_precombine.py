"""Pins for the pre-combined messages of Sec. 6 (gradients of workers that
share a machine are added before they are sent) in oracle/bsgd_oracle.py."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import brute
from oracle import bsgd_oracle as orc

HY = {
    "sgd": dict(opt="sgd", lr=0.1, momentum=0.0, decay=0.0, eps=0.0, clip_norm=0.0),
    "momentum": dict(opt="momentum", lr=0.05, momentum=0.9, decay=0.0, eps=0.0, clip_norm=0.0),
    "rmsprop_mom": dict(opt="rmsprop_mom", lr=0.045, momentum=0.9, decay=0.9, eps=1e-3, clip_norm=0.0),
}


def _tensors(P, opt, seed=0):
    r = np.random.default_rng(seed)
    ns = {"sgd": 0, "momentum": 1, "rmsprop_mom": 2}[opt]
    return [dict(theta=r.standard_normal(P), s0=np.zeros(P) if ns > 0 else None, s1=np.zeros(P) if ns > 1 else None,
                 grad_offset=0)]


def _draw(W, P, seed):
    r = np.random.default_rng(seed)
    return (r.standard_normal((W, P)) * 0.01).astype(np.float32), (1 + r.exponential(1.0, W)).astype(np.float32)


def test_groups_of_one_change_nothing():
    g, t = _draw(7, 33, 1)
    comb, when, cnt = orc.precombine(g, t, [1] * 7)
    assert np.array_equal(comb, g.astype(np.float64)) and np.array_equal(when, t) and cnt.tolist() == [1] * 7
    a, b = _tensors(33, "rmsprop_mom"), _tensors(33, "rmsprop_mom")
    orc.step(g, t, 5, 2, a, HY["rmsprop_mom"])
    orc.step(comb, when, 5, 2, b, dict(HY["rmsprop_mom"], row_count=cnt))
    for k in ("theta", "s0", "s1"):
        assert np.array_equal(a[0][k], b[0][k])


def test_combined_message_is_the_sum_and_leaves_with_the_last_worker():
    g = np.array([[1, 2], [10, 20], [100, 200], [1000, 2000], [5, 5]], np.float32)
    t = np.array([3.0, 1.0, 2.0, 9.0, 4.0], np.float32)
    comb, when, cnt = orc.precombine(g, t, [2, 1, 2])
    assert comb.tolist() == [[11, 22], [100, 200], [1005, 2005]]
    assert when.tolist() == [3.0, 2.0, 9.0] and cnt.tolist() == [2, 1, 2]
    t[3] = np.nan                                        # that worker never finishes
    _, when, _ = orc.precombine(g, t, [2, 1, 2])
    assert when[2] == np.inf
    with pytest.raises(ValueError):
        orc.precombine(g, t, [2, 2])
    with pytest.raises(ValueError):
        orc.precombine(g, t, [5, 0])


def test_mean_divides_by_the_number_of_worker_gradients_hand_worked():
    # machines with 1 and 3 workers; every worker's gradient is 2 -> rows 2 and 6, mean over 4 gradients = 2
    rows = np.array([[2.0], [6.0], [50.0]], np.float32)
    tz = [dict(theta=np.array([1.0]), s0=None, s1=None, grad_offset=0)]
    ok, sel, _ = orc.step(rows, np.array([1.0, 2.0, 3.0], np.float32), 2, 1, tz,
                          dict(HY["sgd"], lr=0.5, row_count=[1, 3, 7]))
    assert ok and sel.tolist() == [0, 1]
    assert tz[0]["theta"][0] == 1.0 - 0.5 * 2.0


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
def test_no_backups_equals_the_plain_mean_over_all_workers(opt):
    W, P = 12, 40
    g, t = _draw(W, P, 2)
    comb, when, cnt = orc.precombine(g, t, [3, 1, 4, 2, 2])
    a, b = _tensors(P, opt), _tensors(P, opt)
    th0 = a[0]["theta"].copy()
    orc.step(comb, when, 5, 0, a, dict(HY[opt], row_count=cnt))
    orc.step(g, t, W, 0, b, HY[opt])
    np.testing.assert_allclose(a[0]["theta"], b[0]["theta"], rtol=0, atol=1e-15)
    if opt == "sgd":
        np.testing.assert_allclose(a[0]["theta"], th0 - 0.1 * np.mean(g.astype(np.float64), axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("seed", range(4))
def test_uniform_groups_equal_the_step_on_the_workers_with_their_machines_time(seed):
    gsz, M, keep, P = 3, 6, 4, 25
    W = gsz * M
    g, t = _draw(W, P, 10 + seed)
    comb, when, cnt = orc.precombine(g, t, [gsz] * M)
    a, b = _tensors(P, "momentum", seed), _tensors(P, "momentum", seed)
    ok, sel, t_step = orc.step(comb, when, keep, M - keep, a, dict(HY["momentum"], row_count=cnt))
    t_machine = np.repeat(when, gsz)                     # every worker waits for its machine
    ok2, sel2, t_step2 = orc.step(g, t_machine, keep * gsz, (M - keep) * gsz, b, HY["momentum"])
    assert ok and ok2 and t_step == t_step2
    assert sorted(sel2.tolist()) == sorted(w for m in sel for w in range(m * gsz, (m + 1) * gsz))
    np.testing.assert_allclose(a[0]["theta"], b[0]["theta"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(a[0]["s0"], b[0]["s0"], rtol=0, atol=1e-15)


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("clip", [0.0, 0.004])
def test_exact_replay_with_uneven_machines(opt, clip):
    sizes = [2, 1, 3, 1]
    W, P, keep = sum(sizes), 5, 3
    g, t = _draw(W, P, 21)
    hy = dict(HY[opt], clip_norm=clip)
    comb, when, cnt = orc.precombine(g, t, sizes)
    tz = _tensors(P, opt, 5)
    th = [Fraction(float(x)) for x in tz[0]["theta"]]
    st = {}
    if opt == "momentum":
        st["v"] = [Fraction(0)] * P
    if opt == "rmsprop_mom":
        st["ms"], st["m"] = [Fraction(0)] * P, [Fraction(0)] * P
    ok, sel, _ = orc.step(comb, when, keep, len(sizes) - keep, tz, dict(hy, row_count=cnt))
    assert ok
    machines = brute.ps_collect(when, keep)              # the collect loop, on machine messages
    assert sorted(machines) == sel.tolist()
    starts = np.concatenate([[0], np.cumsum(sizes)])
    workers = [w for m in machines for w in range(starts[m], starts[m + 1])]
    brute.exact_step(g, workers, th, st, hy)             # exact mean over those workers' own gradients
    for i in range(P):
        assert abs(float(th[i]) - tz[0]["theta"][i]) <= 1e-14 * max(1.0, abs(float(th[i])))


def test_per_worker_clip_of_a_combined_message_is_refused():
    g, t = _draw(4, 6, 3)
    comb, when, cnt = orc.precombine(g, t, [2, 2])
    with pytest.raises(ValueError):
        orc.step(comb, when, 1, 1, _tensors(6, "sgd"), dict(HY["sgd"], worker_clip_norm=1.0, row_count=cnt))
