"""bsgd_step_noalloc: the step on the library's own static device scratch, for
callers that cannot allocate.  Through the C ABI it must leave exactly the bits
bsgd_step leaves (same kernels, only the scratch lives elsewhere), also on a
second, smaller call that finds the first call's leftovers in the scratch."""
import ctypes

import numpy as np
import pytest

from test_gpu_edge import Case

pytestmark = pytest.mark.gpu


def _pair(N, b, layout, opt, seed, hyper=None, ema=None):
    return (Case(N, b, layout, opt, seed=seed, theta_shift=1, hyper=hyper, ema=ema),
            Case(N, b, layout, opt, seed=seed, theta_shift=1, hyper=hyper, ema=ema))


def _noalloc_step(c, g, t):
    """One step of case `c` through the raw C entry point; returns (status, t_step)."""
    import torch
    import paper_1604_00981_amd as bs
    lib = bs.load_library()
    g_dev = torch.from_numpy(g).cuda()
    t_dev = torch.from_numpy(t).cuda()
    st = torch.full((1,), -99, dtype=torch.int32, device="cuda")
    ts = torch.full((1,), -99.0, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream or None
    rc = lib.bsgd_step_noalloc(g_dev.data_ptr(), c.ld, t_dev.data_ptr(), c.N, c.b, c.tensors, len(c.tensors),
                               ctypes.byref(c.hyper), st.data_ptr(), ts.data_ptr(), stream)
    assert rc == bs.BSGD_OK, bs.strerror(rc)
    torch.cuda.synchronize()
    return int(st.item()), float(ts.item())


def _run_pair(ref, dut, steps, sigma=0.01):
    for _ in range(steps):
        g, t = ref.draw(sigma=sigma)
        dut.r = ref.r
        assert ref.both(g, t) == 0                      # bsgd_step with a caller workspace, checked against the oracle
        status, t_step = _noalloc_step(dut, g, t)
        assert status == 0
        assert np.float32(t_step) == np.float32(ref.bs.bsgd_last_status(ref.ws)[1])
    ref.compare()                                       # the existing entry point against the oracle ...
    ga, gb = ref.gpu_arrays(), dut.gpu_arrays()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k          # ... and the new one bit for bit against the existing one


def test_two_calls_in_a_row_the_second_smaller():
    import paper_1604_00981_amd as bs
    # first: 1.2 M columns in 40 tensors with a gap, clipped by the global norm after each worker's own clip,
    # momentum and a moving average: selection, tensor table, per-row and per-chunk partial sums and the stored
    # mean all live in the scratch
    r = np.random.default_rng(3)
    cuts = np.sort(r.choice(np.arange(1, 1_200_000), 39, replace=False))
    sizes = [int(x) for x in np.diff(np.concatenate([[0], cuts, [1_200_000]]))]
    layout, o = [], 3
    for j, n in enumerate(sizes):
        layout.append((o, n))
        o += n + (1000 if j == 20 else 0)
    big_hyper = dict(clip_norm=0.004, worker_clip_norm=9.0)
    ref, dut = _pair(12, 3, layout, "momentum", 81, hyper=big_hyper, ema=0.9)
    assert bs.bsgd_workspace_bytes(ref.span, 12, 3, len(layout), ref.hyper) <= bs.BSGD_STATIC_SCRATCH_BYTES
    _run_pair(ref, dut, steps=2)
    assert bs.bsgd_last_clip(ref.ws)[1] < 1.0
    # second: a much smaller step of another shape (fewer rows, fewer tensors, other optimizer) right after it
    ref2, dut2 = _pair(5, 2, [(1, 30011), (30012, 5), (30017, 901)], "rmsprop_mom", 82, hyper=dict(clip_norm=0.002))
    _run_pair(ref2, dut2, steps=2)
    # and the large one again, on the state it had reached
    _run_pair(ref, dut, steps=1)


def test_too_few_arrivals_and_limits():
    import torch
    import paper_1604_00981_amd as bs
    lib = bs.load_library()
    ref, dut = _pair(4, 2, [(0, 5000), (5000, 1501)], "rmsprop_mom", 83)
    g, t = ref.draw()
    before = dut.gpu_arrays()
    bad = t.copy()
    bad[[0, 2, 5]] = [np.inf, np.nan, np.inf]           # 3 of 6 arrive, N = 4
    status, _ = _noalloc_step(dut, g, bad)
    assert status == bs.BSGD_ERR_TOO_FEW
    after = dut.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    _run_pair(ref, dut, steps=1)                        # the next good step works
    # a clipped step too large for the static scratch is refused on the host with its own code; nothing runs
    A = 0x1000
    P = 20_000_000
    hy = bs.make_hyper("sgd", 0.1, clip_norm=1.0)
    assert bs.bsgd_workspace_bytes(P, 4, 1, 1, hy) > bs.BSGD_STATIC_SCRATCH_BYTES
    tz = bs.make_tensors([(A, None, None, 0, P)])
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert lib.bsgd_step_noalloc(A, P, A, 4, 1, tz, 1, ctypes.byref(hy), st.data_ptr(), None, None) == bs.BSGD_ERR_SCRATCH
    assert "scratch" in bs.strerror(bs.BSGD_ERR_SCRATCH)
    # without clipping the same size fits, and a missing status pointer is an argument error
    hy0 = bs.make_hyper("sgd", 0.1)
    assert bs.bsgd_workspace_bytes(P, 4, 1, 1, hy0) <= bs.BSGD_STATIC_SCRATCH_BYTES
    assert lib.bsgd_step_noalloc(A, P, A, 4, 1, tz, 1, ctypes.byref(hy0), None, None, None) == bs.BSGD_ERR_ARG


def test_recorded_into_a_graph_and_replayed():
    # what the entry point is for: a capture may not allocate, and this call does not.  The first call on the device
    # (which looks the scratch array's address up) has happened above or happens here, before the capture.
    import torch
    import paper_1604_00981_amd as bs
    lib = bs.load_library()
    layout = [(3, 9001), (9004, 17), (9100, 20000)]
    ref, dut = _pair(7, 3, layout, "momentum", 84, hyper=dict(clip_norm=0.01), ema=0.99)
    warm = Case(7, 3, layout, "momentum", seed=85, theta_shift=1, hyper=dict(clip_norm=0.01), ema=0.99)
    g, t = warm.draw()
    assert _noalloc_step(warm, g, t)[0] == 0
    g_dev = torch.zeros((dut.W, dut.ld), device="cuda")
    t_dev = torch.zeros(dut.W, device="cuda")
    st = torch.full((1,), -99, dtype=torch.int32, device="cuda")
    ts = torch.zeros(1, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stream = torch.cuda.current_stream().cuda_stream
        rc = lib.bsgd_step_noalloc(g_dev.data_ptr(), dut.ld, t_dev.data_ptr(), dut.N, dut.b, dut.tensors,
                                   len(dut.tensors), ctypes.byref(dut.hyper), st.data_ptr(), ts.data_ptr(), stream)
    assert rc == bs.BSGD_OK
    for rep in range(3):
        g, t = ref.draw()
        g_dev.copy_(torch.from_numpy(g))
        t_dev.copy_(torch.from_numpy(t))
        graph.replay()
        assert ref.both(g, t) == 0                      # eager bsgd_step between the replays, checked against the oracle
        torch.cuda.synchronize()
        assert int(st.item()) == 0 and np.float32(ts.item()) == np.float32(ref.bs.bsgd_last_status(ref.ws)[1])
        ga, gb = ref.gpu_arrays(), dut.gpu_arrays()
        for k in ga:
            assert np.array_equal(ga[k], gb[k]), (rep, k)
    ref.compare()
