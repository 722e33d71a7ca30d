"""GPU parity for messages pre-combined per machine (Sec. 6 of the paper):
bsgd_precombine and bsgd_step_ex with row_count, through the C ABI, against
the CPU oracle's own pipeline (which never sees a value from the GPU)."""
import numpy as np
import pytest

from oracle import bsgd_oracle as orc
from test_gpu_edge import Case, OPTS

pytestmark = pytest.mark.gpu


def _combine_gpu(g, t, sizes, cols, ld_out=None):
    import torch
    import paper_1604_00981_amd as bs
    W, ld = g.shape
    M = len(sizes)
    ld_out = ld if ld_out is None else ld_out
    gd, td = torch.from_numpy(g).cuda(), torch.from_numpy(t).cuda()
    comb = torch.full((M, ld_out), 7.0, device="cuda")
    when = torch.zeros(M, device="cuda")
    cnt = torch.zeros(M, dtype=torch.int32, device="cuda")
    bs.bsgd_precombine(gd, ld, cols, td, sizes, comb, ld_out, when, cnt)
    torch.cuda.synchronize()
    return comb, when, cnt


@pytest.mark.parametrize("cols,ld,ld_out", [(1, 4, 4), (5, 8, 12), (8192, 8192, 8192), (20011, 20012, 20480),
                                            (70001, 70004, 70004)])
@pytest.mark.parametrize("sizes", [[3, 1, 4, 2, 1, 5], [5, 4, 7], [1] * 16, [16]],
                         ids=["small-machines", "large-machines", "one-worker-each", "one-machine"])
def test_precombine_against_the_oracle(cols, ld, ld_out, sizes):
    # machines of up to three workers on average and larger ones take different launch shapes
    r = np.random.default_rng(cols)
    W = sum(sizes)
    g = np.zeros((W, ld), np.float32)
    g[:, :cols] = (r.standard_normal((W, cols)) * 0.01).astype(np.float32)
    g[:, cols:] = np.nan                                         # padding of the rows is never combined into the result
    t = (1 + r.exponential(1.0, W)).astype(np.float32)
    t[4] = np.nan                                                # a worker of machine 2 never finishes
    t[10] = np.inf
    comb, when, cnt = _combine_gpu(g, t, sizes, cols, ld_out)
    ref, ref_when, ref_cnt = orc.precombine(g[:, :cols], t, sizes)
    assert np.array_equal(when.cpu().numpy(), ref_when)
    assert cnt.cpu().tolist() == ref_cnt.tolist()
    got = comb.cpu().numpy()
    starts = np.concatenate([[0], np.cumsum(sizes)])
    for m in range(len(sizes)):
        bound = sizes[m] * 2.0 ** -24 * np.abs(g[starts[m]:starts[m + 1], :cols].astype(np.float64)).sum(axis=0)
        assert np.all(np.abs(got[m, :cols] - ref[m]) <= bound + 1e-30), m
    cols4 = (cols + 3) // 4 * 4
    assert np.all(got[:, cols4:] == 7.0)                         # nothing is written past the rounded row end


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("clip", [0.0, 0.004])
def test_step_on_combined_messages_matches_the_oracle_pipeline(opt, clip):
    import torch
    import paper_1604_00981_amd as bs
    sizes = [2, 3, 1, 4, 2, 2, 1, 3]                             # 8 machines, 18 workers
    M, keep = len(sizes), 6
    layout = [(0, 9001), (9001, 30), (9040, 12000)]
    c = Case(keep, M - keep, layout, opt, seed=51, hyper=dict(clip_norm=clip), ema=0.9)
    W = sum(sizes)
    r = np.random.default_rng(52)
    for step in range(4):
        g = np.zeros((W, c.ld), np.float32)
        g[:, :c.span] = (r.standard_normal((W, c.span)) * 0.01).astype(np.float32)
        t = (1 + r.exponential(1.0, W)).astype(np.float32)
        comb, when, cnt = _combine_gpu(g, t, sizes, c.span)
        opts = bs.make_select_opts(row_count=cnt)
        bs.bsgd_step_ex(comb, c.ld, when, keep, M - keep, opts, c.tensors, c.hyper, c.ws)
        # the oracle's own pipeline, from the workers' gradients
        o_comb, o_when, o_cnt = orc.precombine(g, t, sizes)
        ok, sel, t_step = orc.step(o_comb, o_when, keep, M - keep, c.otz, dict(c.hy, row_count=o_cnt))
        status, gpu_t_step = bs.bsgd_last_status(c.ws)
        assert ok and status == 0 and np.float32(gpu_t_step) == t_step
        assert bs.bsgd_last_selection(c.ws, keep) == sel.tolist()
        assert bs.bsgd_last_kept_count(c.ws) == keep
        assert bs.bsgd_last_gradient_count(c.ws) == int(sum(sizes[m] for m in sel))
        first = np.concatenate([[0], np.cumsum(sizes)])
        c.account(g, [w for m in sel for w in range(first[m], first[m + 1])])   # the worker gradients the kept messages hold
    c.compare()


def test_rows_that_hold_one_gradient_each_change_nothing():
    import torch
    import paper_1604_00981_amd as bs
    a = Case(7, 2, [(0, 10007)], "rmsprop_mom", seed=53)
    b = Case(7, 2, [(0, 10007)], "rmsprop_mom", seed=53)
    ones = torch.ones(9, dtype=torch.int32, device="cuda")
    for _ in range(2):
        g, t = a.draw()
        a.gpu_step(g, t)
        bs.bsgd_step_ex(torch.from_numpy(g).cuda(), b.ld, torch.from_numpy(t).cuda(), 7, 2,
                        bs.make_select_opts(row_count=ones), b.tensors, b.hyper, b.ws)
    assert bs.bsgd_last_gradient_count(a.ws) == 7 and bs.bsgd_last_gradient_count(b.ws) == 7
    ga, gb = a.gpu_arrays(), b.gpu_arrays()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k


def test_deadline_mode_divides_by_the_gradients_of_every_message_in_time():
    import torch
    import paper_1604_00981_amd as bs
    c = Case(4, 2, [(0, 5003)], "sgd", seed=54)
    g, _ = c.draw()
    t = np.array([1.0, 5.0, 2.0, 9.0, 3.0, 4.0], np.float32)
    counts = np.array([2, 1, 3, 1, 1, 4], np.int32)
    th0 = c.gpu_arrays()["theta"].astype(np.float64)
    cnt_dev = torch.from_numpy(counts).cuda()                    # must outlive the options that point at it
    opts = bs.make_select_opts(deadline=4.5, n_min=2, row_count=cnt_dev)
    bs.bsgd_step_ex(torch.from_numpy(g).cuda(), c.ld, torch.from_numpy(t).cuda(), 4, 2, opts, c.tensors, c.hyper, c.ws)
    assert bs.bsgd_last_status(c.ws)[0] == 0
    assert bs.bsgd_last_kept_count(c.ws) == 4                    # messages 0, 2, 4, 5 are in time
    assert bs.bsgd_last_gradient_count(c.ws) == 2 + 3 + 1 + 4
    ok, sel, _ = orc.step(g, t, 4, 2, c.otz, dict(c.hy, deadline=4.5, n_min=2, row_count=counts))
    assert ok and sel.tolist() == [0, 2, 4, 5]
    c.account(g, sel)              # a row here stands for counts[k] gradients: the budget below is the smaller, stricter one
    c.compare()
    assert not np.array_equal(th0, c.gpu_arrays()["theta"])


def test_a_kept_row_without_gradients_is_an_error_and_nothing_is_updated():
    import torch
    import paper_1604_00981_amd as bs
    c = Case(3, 1, [(0, 3001)], "momentum", seed=55)
    g, t = c.draw()
    before = c.gpu_arrays()
    kept = orc.select_first_n(t, 3, 1)[0]
    counts = np.full(4, 2, np.int32)
    counts[kept[1]] = 0
    cnt_dev = torch.from_numpy(counts).cuda()
    opts = bs.make_select_opts(row_count=cnt_dev)
    bs.bsgd_step_ex(torch.from_numpy(g).cuda(), c.ld, torch.from_numpy(t).cuda(), 3, 1, opts, c.tensors, c.hyper, c.ws)
    assert bs.bsgd_last_status(c.ws)[0] == bs.BSGD_ERR_ARG
    after = c.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    # a zero count on the dropped row does not matter
    dropped = [w for w in range(4) if w not in kept][0]
    counts[:] = 2
    counts[dropped] = 0
    cnt_dev2 = torch.from_numpy(counts).cuda()
    opts = bs.make_select_opts(row_count=cnt_dev2)
    bs.bsgd_step_ex(torch.from_numpy(g).cuda(), c.ld, torch.from_numpy(t).cuda(), 3, 1, opts, c.tensors, c.hyper, c.ws)
    assert bs.bsgd_last_status(c.ws)[0] == 0 and bs.bsgd_last_gradient_count(c.ws) == 6


def test_refusals():
    import torch
    import paper_1604_00981_amd as bs
    g = torch.zeros((4, 16), device="cuda")
    t = torch.zeros(4, device="cuda")
    out = torch.zeros((2, 16), device="cuda")
    when = torch.zeros(2, device="cuda")
    cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
    ok = lambda **kw: bs.bsgd_precombine(kw.get("g", g), kw.get("ld", 16), kw.get("cols", 13), t, kw.get("sizes", [1, 3]),
                                          kw.get("out", out), kw.get("ld_out", 16), when, cnt)
    ok()
    for bad in (dict(sizes=[]), dict(sizes=[0, 4]), dict(sizes=[200, 100]), dict(ld=14), dict(ld_out=12), dict(cols=0),
                dict(cols=17), dict(out=g), dict(out=g[1:3]), dict(g=g.view(-1)[1:].view(-1))):
        with pytest.raises(bs.BsgdError):
            ok(**bad)
    # the selection alone has nowhere to put the divisor
    sel = torch.zeros(4, dtype=torch.int32, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    nk = torch.zeros(1, dtype=torch.int32, device="cuda")
    ones = torch.ones(4, dtype=torch.int32, device="cuda")
    with pytest.raises(bs.BsgdError):
        bs.bsgd_select_ex(t, 3, 1, bs.make_select_opts(row_count=ones), sel, nk, None, st)
    # per-worker clipping of a combined message
    c = Case(3, 1, [(0, 100)], "sgd", seed=56, hyper=dict(worker_clip_norm=1.0))
    with pytest.raises(bs.BsgdError):
        bs.bsgd_step_ex(torch.zeros((4, c.ld), device="cuda"), c.ld, t, 3, 1, bs.make_select_opts(row_count=ones),
                        c.tensors, c.hyper, c.ws)
