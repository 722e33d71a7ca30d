"""A step only enqueues kernels on the caller's stream (descriptors travel in
kernel arguments, nothing is copied from the host, nothing is allocated), so
it can be recorded into a HIP graph.  A recorded step is replayed several
times on fresh inputs, with eager work and synchronisation in between, and
every replay must leave exactly the bits the eager call leaves."""
import numpy as np
import pytest

from test_gpu_edge import Case

pytestmark = pytest.mark.gpu

KINDS = {
    "single_rmsprop": dict(N=9, b=2, layout=[(0, 30011)], opt="rmsprop_mom", hyper=None, ema=None),
    "multi_clipped_momentum_ema": dict(N=7, b=3, layout=[(3, 9001), (9004, 17), (9100, 20000)], opt="momentum",
                                       hyper=dict(clip_norm=0.01), ema=0.99),
    "multi_worker_clip_sgd": dict(N=5, b=1, layout=[(0, 4097), (4097, 4099)], opt="sgd",
                                  hyper=dict(worker_clip_norm=0.5), ema=None),
}


@pytest.mark.parametrize("kind", sorted(KINDS))
def test_recorded_step_replays_like_the_eager_call(kind):
    import torch
    import paper_1604_00981_amd as bs
    k = KINDS[kind]
    mk = lambda seed: Case(k["N"], k["b"], k["layout"], k["opt"], seed=seed, hyper=k["hyper"], ema=k["ema"])
    eager, rec, scratch = mk(31), mk(31), mk(32)
    for a, b in zip(eager.gpu_arrays().values(), rec.gpu_arrays().values()):
        assert np.array_equal(a, b)

    g_dev = torch.zeros((rec.W, rec.ld), device="cuda")
    t_dev = torch.zeros(rec.W, device="cuda")
    # once eagerly on throw-away state, so that one-time set-up is not part of the recording
    scratch.gpu_step(*scratch.draw())
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bs.bsgd_step(g_dev, rec.ld, t_dev, rec.N, rec.b, rec.tensors, rec.hyper, rec.ws)
    # recording runs nothing
    for a, b in zip(eager.gpu_arrays().values(), rec.gpu_arrays().values()):
        assert np.array_equal(a, b)

    for rep in range(4):
        g, t = eager.draw()
        g_dev.copy_(torch.from_numpy(g))
        t_dev.copy_(torch.from_numpy(t))
        graph.replay()
        eager.both(g, t)                                # eager step (checked against the oracle's selection) ...
        torch.cuda.synchronize()                        # ... and a synchronisation between replays
        assert bs.bsgd_last_status(rec.ws)[0] == 0
        assert bs.bsgd_last_selection(rec.ws, rec.N) == bs.bsgd_last_selection(eager.ws, eager.N)
        ga, gb = eager.gpu_arrays(), rec.gpu_arrays()
        for name in ga:
            assert np.array_equal(ga[name], gb[name]), (rep, name)
    eager.compare()


def test_recorded_step_with_too_few_arrivals_touches_nothing():
    import torch
    import paper_1604_00981_amd as bs
    c = Case(6, 2, [(0, 5003)], "momentum", seed=33)
    warm = Case(6, 2, [(0, 5003)], "momentum", seed=34)
    warm.gpu_step(*warm.draw())
    torch.cuda.synchronize()
    g, t = c.draw()
    g_dev = torch.from_numpy(g).cuda()
    t_dev = torch.from_numpy(t).cuda()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bs.bsgd_step(g_dev, c.ld, t_dev, c.N, c.b, c.tensors, c.hyper, c.ws)
    before = c.gpu_arrays()
    bad = t.copy()
    bad[:3] = np.inf                                    # only 5 of the 6 needed ever arrive
    t_dev.copy_(torch.from_numpy(bad))
    graph.replay()
    torch.cuda.synchronize()
    assert bs.bsgd_last_status(c.ws)[0] == bs.BSGD_ERR_TOO_FEW
    after = c.gpu_arrays()
    for name in before:
        assert np.array_equal(before[name], after[name]), name
    t_dev.copy_(torch.from_numpy(t))                    # the same recording works again once enough arrive
    graph.replay()
    torch.cuda.synchronize()
    assert bs.bsgd_last_status(c.ws)[0] == 0
    assert not np.array_equal(before["theta"], c.gpu_arrays()["theta"])
