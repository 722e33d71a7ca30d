"""GPU edge cases and properties of the step, through the C ABI, checked
against the CPU oracle or against properties that need no oracle."""
import numpy as np
import pytest

from harness import ELEM_FACTOR, REL_L2_TOL
from oracle import bsgd_oracle as orc

pytestmark = pytest.mark.gpu

OPTS = {
    "sgd": dict(opt="sgd", lr=0.1, momentum=0.0, decay=0.0, eps=0.0, clip_norm=0.0),
    "momentum": dict(opt="momentum", lr=0.05, momentum=0.9, decay=0.0, eps=0.0, clip_norm=0.0),
    "rmsprop_mom": dict(opt="rmsprop_mom", lr=0.045, momentum=0.9, decay=0.9, eps=1e-3, clip_norm=0.0),
}
NS = {"sgd": 0, "momentum": 1, "rmsprop_mom": 2}


def _f32(h):
    return {k: (v if k == "opt" else float(np.float32(v))) for k, v in h.items()}


class Case:
    """A small ad-hoc problem living on the GPU, with a matching fp64 oracle copy.

    layout: list of (grad_offset, numel); theta_shift: element offset of every
    tensor's theta/state view inside its own allocation (to misalign them)."""

    def __init__(self, N, b, layout, opt, seed=0, ld=None, theta_shift=0, hyper=None, ema=None):
        import torch
        import paper_1604_00981_amd as bs
        self.bs, self.torch = bs, torch
        self.N, self.b, self.W = N, b, N + b
        self.layout, self.opt = layout, opt
        self.hy = _f32(dict(OPTS[opt], ema_decay=(ema or 0.0), **(hyper or {})))
        self.use_ema = ema is not None
        r = np.random.default_rng(seed)
        self.r = r
        span = max([o + n for o, n in layout] + [0])
        self.span = span
        self.ld = ((span + 3) // 4 * 4) if ld is None else ld
        ns = NS[opt]
        self.th, self.s = [], [[] for _ in range(ns)]
        self.ema = []
        self.otz = []
        for o, n in layout:
            t0 = (r.standard_normal(n) * 0.05).astype(np.float32)
            buf = torch.zeros(n + theta_shift, device="cuda")
            buf[theta_shift:] = torch.from_numpy(t0).cuda()
            self.th.append(buf[theta_shift:])
            for i in range(ns):
                self.s[i].append(torch.zeros(n + theta_shift, device="cuda")[theta_shift:])
            if self.use_ema:
                ebuf = torch.zeros(n + theta_shift, device="cuda")
                ebuf[theta_shift:] = torch.from_numpy(t0).cuda()
                self.ema.append(ebuf[theta_shift:])
            self.otz.append(dict(theta=t0.astype(np.float64), s0=np.zeros(n) if ns > 0 else None,
                                 s1=np.zeros(n) if ns > 1 else None, grad_offset=o,
                                 ema=t0.astype(np.float64) if self.use_ema else None))
        self.tensors = bs.make_tensors([(self.th[j], self.s[0][j] if ns > 0 else None,
                                         self.s[1][j] if ns > 1 else None, o, n,
                                         self.ema[j] if self.use_ema else None)
                                        for j, (o, n) in enumerate(layout)])
        self.hyper = bs.make_hyper(**self.hy)
        self.ws = bs.alloc_workspace(span, N, b, len(layout), self.hyper)
        # per element of theta (tensors concatenated): sum over steps and kept workers of |g|
        self.abs_sum = np.zeros(sum(n for _, n in layout))
        self.max_kept = N
        self.accounted = False
        self.steps = 0

    def draw(self, sigma=0.01, bias=0.0):
        g = np.zeros((self.W, self.ld), np.float32)
        g[:, :self.span] = (bias + self.r.standard_normal((self.W, self.span)) * sigma).astype(np.float32)
        t = (1.0 + self.r.exponential(1.0, self.W)).astype(np.float32)
        return g, t

    def gpu_step(self, g, t, opts=None):
        """opts: None (bsgd_step) or a dict with tags / step_tag / deadline / n_min (bsgd_step_ex)."""
        torch, bs = self.torch, self.bs
        self.g_dev = torch.from_numpy(g).cuda()
        t_dev = torch.from_numpy(t).cuda()
        if opts is None:
            bs.bsgd_step(self.g_dev, self.ld, t_dev, self.N, self.b, self.tensors, self.hyper, self.ws)
        else:
            tags = opts.get("tags")
            self.tags_dev = None if tags is None else torch.from_numpy(np.asarray(tags, np.int32)).cuda()
            so = bs.make_select_opts(self.tags_dev, int(opts.get("step_tag", 0)), float(opts.get("deadline", np.inf)),
                                     int(opts.get("n_min", 0)))
            bs.bsgd_step_ex(self.g_dev, self.ld, t_dev, self.N, self.b, so, self.tensors, self.hyper, self.ws)
        return bs.bsgd_last_status(self.ws)

    def both(self, g, t, opts=None):
        status, t_step = self.gpu_step(g, t, opts)
        ok, sel, ots = orc.step(g, t, self.N, self.b, self.otz, dict(self.hy, **(opts or {})))
        assert (status == 0) == ok
        if ok:
            n_kept = len(sel)
            if opts is not None and opts.get("n_min", 0) > 0:
                assert self.bs.bsgd_last_kept_count(self.ws) == n_kept
            assert self.bs.bsgd_last_selection(self.ws, n_kept) == sel.tolist()
            assert np.float32(t_step) == ots
            self.account(g, sel)
        return status

    def account(self, g, rows):
        """Adds |g| of the given gradient rows (those a step just summed) to the per-element error budget."""
        rows = [int(k) for k in rows]
        self.steps += 1
        self.max_kept = max(self.max_kept, len(rows))
        o = 0
        for off, n in self.layout:
            self.abs_sum[o:o + n] += np.abs(g[rows, off:off + n]).sum(axis=0, dtype=np.float64)
            o += n
        self.accounted = True

    def gpu_arrays(self):
        out = {"theta": np.concatenate([x.cpu().numpy() for x in self.th]) if self.th else np.zeros(0)}
        for i, nm in enumerate(("s0", "s1")[:len(self.s)]):
            out[nm] = np.concatenate([x.cpu().numpy() for x in self.s[i]])
        if self.use_ema:
            out["ema"] = np.concatenate([x.cpu().numpy() for x in self.ema])
        return out

    def compare(self):
        """The agreement criteria of the parity harness, on everything this case updated through `both`:
        relative L2 error <= 1e-6 for theta, each state buffer and the moving average (tensors concatenated);
        per element of theta, |gpu - oracle| <= 8 * N * 2^-24 * sum over steps and kept workers of |g|."""
        got = self.gpu_arrays()
        for nm, arr in got.items():
            ref = np.concatenate([t[nm] for t in self.otz])
            err = arr.astype(np.float64) - ref
            den = np.linalg.norm(ref)
            if den > 0:
                rel = np.linalg.norm(err) / den
                assert rel <= REL_L2_TOL, (nm, rel)
            else:
                assert not err.any(), nm
            if nm == "theta":
                assert self.accounted, "compare() needs the steps' gradients (both() or account())"
                # plus what storing theta in fp32 after every step costs whatever the gradients are (half an ulp
                # each time): with few kept rows and millions of elements some element's gradients are all tiny
                # and the first term alone falls below the rounding of the store
                bound = ELEM_FACTOR * self.max_kept * self.abs_sum + self.steps * 2.0 ** -24 * np.abs(ref)
                worst = float(np.max(np.abs(err) / np.maximum(bound, 1e-300))) if err.size else 0.0
                assert worst <= 1.0, f"theta: per-element error is {worst:.3f}x the bound"


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 255, 1023, 1024, 1025, 2047, 4096, 4097, 8191, 12289])
def test_ragged_sizes_single_tensor(opt, P):
    c = Case(5, 2, [(0, P)], opt, seed=P)
    # On a handful of elements the kept gradients of one element can cancel to far below their magnitudes, and the
    # relative error of ANY fp32 sum is then (N-1) 2^-24 sum|g| / |sum g|, unbounded: relative L2 over such a vector
    # measures the input's conditioning, not the kernel.  The tiny sizes therefore draw gradients with a common
    # offset (a well-conditioned mean); from 64 elements on the zero-mean draw is used as everywhere else.
    bias = 0.02 if P < 64 else 0.0
    for _ in range(2):
        c.both(*c.draw(bias=bias))
    c.compare()


@pytest.mark.parametrize("opt", ["sgd", "rmsprop_mom"])
@pytest.mark.parametrize("shift", [0, 1, 2, 3])
@pytest.mark.parametrize("goff", [0, 1, 2, 3, 5])
def test_misaligned_tensor_starts(opt, shift, goff):
    # theta/state start `shift` elements into their allocation, the gradient
    # segment starts `goff` elements into the row: every relative phase occurs
    layout = [(goff, 3001), (goff + 3001, 1), (goff + 3002, 2050), (goff + 5052 + 3, 77)]   # a gap of 3 too
    c = Case(4, 1, layout, opt, seed=10 * shift + goff, theta_shift=shift)
    for _ in range(2):
        c.both(*c.draw())
    c.compare()


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("clip", [0.0, 0.01])
def test_moving_average_edges(opt, clip):
    # unaligned tensors, cut groups, a gap; alpha = 0 checks the index (thetabar = theta before the update)
    layout = [(3, 3001), (3004, 1), (3005, 2050), (5060, 77), (5137, 9000)]
    for alpha in (0.0, 0.9):
        c = Case(4, 1, layout, opt, seed=31, theta_shift=1, hyper=dict(clip_norm=clip), ema=alpha)
        before = None
        for _ in range(2):
            before = c.gpu_arrays()["theta"].copy()
            c.both(*c.draw())
        c.compare()
        if alpha == 0.0:
            assert np.array_equal(c.gpu_arrays()["ema"], before)     # bitwise the pre-update parameters
    # too few arrivals: the average is left alone as well
    g, t = c.draw()
    snap = c.gpu_arrays()
    t[[0, 1, 2]] = np.inf
    assert c.both(g, t) == c.bs.BSGD_ERR_TOO_FEW
    after = c.gpu_arrays()
    for k in snap:
        assert np.array_equal(snap[k], after[k]), k


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
@pytest.mark.parametrize("both", [False, True])
def test_per_worker_clipping(opt, both):
    # every kept gradient clipped by its own global norm (over tensor columns only), then averaged;
    # optionally followed by the clip of the mean
    layout = [(5, 3001), (3006, 1), (3007, 2050), (5070, 77), (5147, 9000)]        # a gap at 5057..5069
    hy = dict(worker_clip_norm=0.9, clip_norm=0.05 if both else 0.0)
    c = Case(9, 3, layout, opt, seed=41, theta_shift=1, hyper=hy)
    for step in range(3):
        g, t = c.draw(sigma=0.01)
        g *= c.r.uniform(0.2, 3.0, (c.W, 1)).astype(np.float32)                    # workers of very different norms
        covered = np.zeros(c.ld, bool)
        for o, n in layout:
            covered[o:o + n] = True
        g[:, ~covered] = 50.0                                                      # gap columns must not enter any norm
        sel, _ = orc.select_first_n(t, c.N, c.b)
        sc = orc.worker_clip_scales(g, sel, [(o, o + n) for o, n in layout], c.hy["worker_clip_norm"])
        assert (sc < 1).any() and (sc == 1).any()                                  # some clipped, some not
        c.both(g, t)
    c.compare()


@pytest.mark.parametrize("opt", ["momentum", "rmsprop_mom"])
@pytest.mark.parametrize("multi", [False, True])
def test_per_worker_clipping_under_a_deadline_that_keeps_more_than_N(opt, multi):
    # Time-outs in place of backups (Sec. 6) together with each worker's own clip (Appendix A.3): with N = 6, b = 4
    # the deadline lets 10, then 8, then 10 messages in, so rows beyond the N-th need their own norm and scale
    layout = [(3, 9001), (9004, 1), (9005, 7050), (16070, 77), (16147, 9000)] if multi else [(0, 20011)]
    N, b = 6, 4
    c = Case(N, b, layout, opt, seed=61, theta_shift=1 if multi else 0, hyper=dict(worker_clip_norm=1.5))
    ranges = [(o, o + n) for o, n in layout]
    seen_clipped = seen_unclipped = False
    for step, want in enumerate((10, 8, 10)):
        g, t = c.draw(sigma=0.01)
        g *= c.r.uniform(0.2, 3.0, (c.W, 1)).astype(np.float32)                    # workers of very different norms
        tau = float(np.sort(t)[want - 1])                                          # exactly `want` messages are in time
        opts = dict(deadline=tau, n_min=2)
        sel, _ = orc.select_ex(t, N, b, deadline=tau, n_min=2)
        assert len(sel) == want > N
        sc = orc.worker_clip_scales(g, sel, ranges, c.hy["worker_clip_norm"])
        seen_clipped |= bool((sc[N:] < 1).any())                                   # among the rows beyond the N-th ...
        seen_unclipped |= bool((sc[N:] == 1).any())
        assert c.both(g, t, opts) == 0
    assert seen_clipped and seen_unclipped                                         # ... some were clipped, some not
    c.compare()
    # the same case run twice leaves the same bits (the per-row partial sums have a slot of their own each)
    d = Case(N, b, layout, opt, seed=61, theta_shift=1 if multi else 0, hyper=dict(worker_clip_norm=1.5))
    for want in (10, 8, 10):
        g, t = d.draw(sigma=0.01)
        g *= d.r.uniform(0.2, 3.0, (d.W, 1)).astype(np.float32)
        d.gpu_step(g, t, dict(deadline=float(np.sort(t)[want - 1]), n_min=2))
    ga, gb = c.gpu_arrays(), d.gpu_arrays()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k


def test_per_worker_clipping_off_when_threshold_is_large():
    a = Case(6, 2, [(0, 7001)], "momentum", seed=42)
    b = Case(6, 2, [(0, 7001)], "momentum", seed=42, hyper=dict(worker_clip_norm=1e9))
    for _ in range(2):
        g, t = a.draw()
        a.gpu_step(g, t)
        b.gpu_step(g, t)
    ga, gb = a.gpu_arrays(), b.gpu_arrays()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k          # a scale of exactly 1 changes no bit


def test_update_in_two_partial_calls_equals_one_call():
    # top-layer tensors can be updated while lower layers are still arriving (Appendix A.3's pipelining):
    # a step applied tensor subset by tensor subset gives the same bits as one call
    import torch
    layout = [(0, 5000), (5000, 777), (5777, 12001), (17778, 64)]
    one = Case(7, 2, layout, "rmsprop_mom", seed=43)
    two = Case(7, 2, layout, "rmsprop_mom", seed=43)
    bs = one.bs
    for _ in range(2):
        g, t = one.draw()
        one.gpu_step(g, t)
        g_dev, t_dev = torch.from_numpy(g).cuda(), torch.from_numpy(t).cuda()
        sel = torch.zeros(7, dtype=torch.int32, device="cuda")
        st = torch.zeros(1, dtype=torch.int32, device="cuda")
        bs.bsgd_select_first_n(t_dev, 7, 2, sel, None, st)
        for part in ([3, 2], [0, 1]):                   # "top layers" first
            items = [(two.th[j], two.s[0][j], two.s[1][j], layout[j][0], layout[j][1]) for j in part]
            bs.bsgd_reduce_update(g_dev, two.ld, sel, st, 7, bs.make_tensors(items), two.hyper, two.ws)
    ga, gb = one.gpu_arrays(), two.gpu_arrays()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), k


def test_tensors_listed_out_of_order_with_gaps():
    # descriptors in arbitrary order, holes between tensors, first tensor not at column 0
    layout = [(9000, 2500), (7, 1000), (4001, 3), (1500, 2501), (4100, 4099), (8300, 64)]
    c = Case(5, 2, layout, "rmsprop_mom", seed=21)
    for _ in range(2):
        g, t = c.draw()
        # poison the gap columns: they belong to no tensor and must not matter
        covered = np.zeros(c.ld, bool)
        for o, n in layout:
            covered[o:o + n] = True
        g[:, ~covered] = np.nan
        c.both(g, t)
    c.compare()
    cc = Case(5, 2, layout, "momentum", seed=22, hyper=dict(clip_norm=0.01))
    for _ in range(2):
        g, t = cc.draw()
        covered = np.zeros(cc.ld, bool)
        for o, n in layout:
            covered[o:o + n] = True
        g[:, ~covered] = 1e3            # finite garbage in the gaps must not enter the norm
        cc.both(g, t)
    cc.compare()


@pytest.mark.parametrize("kind", ["plain", "clip", "worker_clip", "ema_clip"])
@pytest.mark.parametrize("gap", [200_003, 1_100_001])
def test_wide_gaps_between_tensors_are_neither_launched_nor_read(kind, gap):
    # A partial-range update (Appendix A.3: top layers' gradients are sent while the lower layers are still being
    # computed) names only the tensors whose gradients are in.  The columns in between are NaN here: no chunk that
    # lies wholly in a gap may be read, in any launch shape.  The narrow gap stays inside one run of chunks in the
    # wide shapes (its workgroups stand down on the device), the wide one splits the call into two runs.
    import paper_1604_00981_amd as bs
    hyper = dict(plain={}, clip=dict(clip_norm=0.004), worker_clip=dict(worker_clip_norm=1.4),
                 ema_clip=dict(clip_norm=0.004))[kind]
    layout = [(5, 30_001), (30_006, 2_000), (32_006 + gap, 20_003)]
    shapes = [bs.bsgd_get_shape(i) for i in range(bs.bsgd_num_shapes())]
    results = []
    try:
        for shape in shapes:
            bs.bsgd_set_tuning(*shape)
            c = Case(6, 2, layout, "rmsprop_mom" if kind != "worker_clip" else "momentum", seed=91, theta_shift=1,
                     hyper=hyper, ema=0.9 if kind == "ema_clip" else None)
            covered = np.zeros(c.ld, bool)
            for o, n in layout:
                covered[o:o + n] = True
            for _ in range(2):
                g, t = c.draw()
                g *= c.r.uniform(0.3, 3.0, (c.W, 1)).astype(np.float32)
                g[:, ~covered] = np.nan
                assert c.both(g, t) == 0
            c.compare()
            chunk_cols = 4 * shape[0] * shape[1]
            passes = {"plain": 1, "clip": 2, "worker_clip": 2, "ema_clip": 2}[kind]
            if gap // chunk_cols > 64 + 1:
                assert bs.bsgd_last_launch_count() == 2 * passes      # one launch per run and pass: the gap is not launched
            else:
                assert bs.bsgd_last_launch_count() == passes          # one run; gap chunks stand down on the device
            results.append(c.gpu_arrays())
    finally:
        bs.bsgd_set_tuning()
    if kind == "plain":
        for a, bb in zip(results, results[1:]):
            for k in a:
                assert np.array_equal(a[k], bb[k]), k


def test_many_tensors_multiple_upload_batches_and_empty_ones():
    r = np.random.default_rng(5)
    sizes = [int(x) for x in r.integers(0, 700, 333)]          # some are empty
    sizes[0], sizes[-1], sizes[100] = 0, 0, 9000
    layout, o = [], 0
    for n in sizes:
        layout.append((o, n))
        o += n
    c = Case(6, 2, layout, "rmsprop_mom", seed=6)
    for _ in range(2):
        c.both(*c.draw())
    c.compare()


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
def test_clipped_step_matches_oracle_multi_tensor(opt):
    layout = [(0, 5000), (5000, 3), (5003, 1200), (6203, 4097)]
    c = Case(7, 2, layout, opt, seed=3, hyper=dict(clip_norm=0.01))
    for i in range(3):
        g, t = c.draw(sigma=0.01)
        c.both(g, t)
        nrm, scale = c.bs.bsgd_last_clip(c.ws)
        sel, _ = orc.select_first_n(t, c.N, c.b)
        G = [orc.reduce_mean(g, sel, o, o + n) for o, n in layout]
        ref_nrm = float(np.sqrt(sum(np.dot(x, x) for x in G)))
        assert nrm == pytest.approx(ref_nrm, rel=1e-6)
        assert scale == pytest.approx(orc.clip_scale(G, c.hy["clip_norm"]), rel=1e-6)
        assert scale < 1.0
    c.compare()


def test_clip_threshold_above_norm_changes_nothing():
    layout = [(0, 3000)]
    a = Case(4, 1, layout, "momentum", seed=8)
    b = Case(4, 1, layout, "momentum", seed=8, hyper=dict(clip_norm=1e6))
    for _ in range(2):
        g, t = a.draw()
        b.r = a.r
        a.gpu_step(g, t)
        b.gpu_step(g, t)
        nrm, scale = b.bs.bsgd_last_clip(b.ws)
        assert scale == 1.0
    ga, gb = a.gpu_arrays(), b.gpu_arrays()
    for k in ga:
        # the two-pass path stores the fp32 mean and multiplies it by a scale of exactly 1: the same bits
        assert np.array_equal(ga[k], gb[k]), k


@pytest.mark.parametrize("opt", ["sgd", "momentum", "rmsprop_mom"])
def test_too_few_arrivals_leaves_theta_and_state_untouched(opt):
    c = Case(4, 2, [(0, 5000), (5000, 1501)], opt, seed=11)
    g, t = c.draw()
    assert c.both(g, t) == 0
    before = c.gpu_arrays()
    t_bad = t.copy()
    t_bad[[0, 2, 5]] = [np.inf, np.nan, np.inf]                # only 3 of 6 arrive, N = 4
    assert c.both(g, t_bad) == c.bs.BSGD_ERR_TOO_FEW
    after = c.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    # and with clipping on (three kernels must all stand down)
    cc = Case(4, 2, [(0, 5000)], opt, seed=12, hyper=dict(clip_norm=0.001))
    g, t = cc.draw()
    cc.both(g, t)
    before = cc.gpu_arrays()
    assert cc.both(g, t_bad) == cc.bs.BSGD_ERR_TOO_FEW
    after = cc.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    # the next good step works again
    assert cc.both(*cc.draw()) == 0
    cc.compare()


@pytest.mark.parametrize("opt", ["sgd", "rmsprop_mom"])
def test_dropped_rows_are_never_read(opt):
    # NaN in dropped rows must not reach theta: bitwise equal to zero-filled rows
    a = Case(5, 3, [(0, 9001)], opt, seed=13)
    b = Case(5, 3, [(0, 9001)], opt, seed=13)
    for _ in range(2):
        g, t = a.draw()
        b.r = a.r
        sel, _ = orc.select_first_n(t, 5, 3)
        dropped = [k for k in range(8) if k not in set(sel.tolist())]
        g_nan, g_zero = g.copy(), g.copy()
        g_nan[dropped] = np.nan
        g_zero[dropped] = 0.0
        a.gpu_step(g_nan, t)
        b.gpu_step(g_zero, t)
    ga, gb = a.gpu_arrays(), b.gpu_arrays()
    for k in ga:
        assert np.isfinite(ga[k]).all()
        assert np.array_equal(ga[k], gb[k]), k


def test_worker_permutation():
    N, b, P = 9, 4, 6001
    a = Case(N, b, [(0, P)], "momentum", seed=14)
    p = Case(N, b, [(0, P)], "momentum", seed=14)
    g, t = a.draw()
    perm = np.random.default_rng(1).permutation(N + b)
    a.gpu_step(g, t)
    p.gpu_step(np.ascontiguousarray(g[perm]), np.ascontiguousarray(t[perm]))
    sel_a = a.bs.bsgd_last_selection(a.ws, N)
    sel_p = p.bs.bsgd_last_selection(p.ws, N)
    assert sorted(int(perm[j]) for j in sel_p) == sel_a
    ga, gp = a.gpu_arrays(), p.gpu_arrays()
    # same set, different summation order: equal up to fp32 rounding of the sum
    np.testing.assert_allclose(gp["theta"], ga["theta"], rtol=1e-6, atol=1e-9)


def test_b0_keeps_everyone_and_equals_plain_mean_update():
    c = Case(6, 0, [(0, 4099)], "sgd", seed=15)
    g, t = c.draw()
    th0 = c.gpu_arrays()["theta"].astype(np.float64)
    c.gpu_step(g, t)
    assert c.bs.bsgd_last_selection(c.ws, 6) == list(range(6))
    ref = th0 - c.hy["lr"] * g[:, :4099].astype(np.float64).mean(axis=0)
    np.testing.assert_allclose(c.gpu_arrays()["theta"], ref, rtol=1e-6, atol=1e-9)


def test_run_to_run_determinism_and_checkpoint_resume():
    def run(split_at=None):
        c = Case(10, 3, [(1, 7001), (7002, 333)], "rmsprop_mom", seed=16)
        for i in range(6):
            g, t = c.draw()
            if split_at is not None and i == split_at:
                # checkpoint: copy everything out, into fresh buffers, and go on
                snap = c.gpu_arrays()
                c2 = Case(10, 3, [(1, 7001), (7002, 333)], "rmsprop_mom", seed=99)
                o = 0
                for j, (_, n) in enumerate(c.layout):
                    c2.th[j].copy_(c.torch.from_numpy(snap["theta"][o:o + n]))
                    c2.s[0][j].copy_(c.torch.from_numpy(snap["s0"][o:o + n]))
                    c2.s[1][j].copy_(c.torch.from_numpy(snap["s1"][o:o + n]))
                    o += n
                c2.r = c.r
                c = c2
            c.gpu_step(g, t)
        return c.gpu_arrays()

    a, b, r = run(), run(), run(split_at=3)
    for k in a:
        assert np.array_equal(a[k], b[k]), k            # bitwise repeatable
        assert np.array_equal(a[k], r[k]), k            # state is entirely caller-owned


def test_every_compiled_launch_shape_gives_identical_bits():
    import paper_1604_00981_amd as bs
    shapes = [bs.bsgd_get_shape(i) for i in range(bs.bsgd_num_shapes())]
    results = []
    try:
        for shape in shapes:
            bs.bsgd_set_tuning(*shape)
            c = Case(23, 3, [(2, 20011), (20013, 5), (20018, 4100)], "rmsprop_mom", seed=17, hyper=dict(clip_norm=0.0))
            for _ in range(2):
                c.both(*c.draw())
            c.compare()                                 # every shape against the oracle, not only against each other
            cc = Case(23, 3, [(2, 20011), (20013, 5), (20018, 4100)], "momentum", seed=18, hyper=dict(clip_norm=0.002))
            for _ in range(2):
                cc.both(*cc.draw())
            cc.compare()
            results.append((c.gpu_arrays(), cc.gpu_arrays()))
    finally:
        bs.bsgd_set_tuning()                          # back to the automatic choice
    for (a, ac), (b, bc) in zip(results, results[1:]):
        for k in a:
            assert np.array_equal(a[k], b[k]), k        # rows are added in the same order in every shape
        # the clipped norm is summed per block, so block shape may move its last bits
        for k in ac:
            np.testing.assert_allclose(ac[k], bc[k], rtol=1e-6, atol=1e-9)


# What each compiled launch shape must also be compared with the oracle on (beside the two cases above): every
# kernel instantiation a full-size call can reach.  Layouts span several chunks of the widest shape (8192 columns),
# with a chunk inside one tensor, chunks holding tensor boundaries, cut groups, a gap and a ragged end.
_WIDE_MULTI = [(2, 40011), (40013, 5), (40018, 4100), (44200, 9000)]
_INSTANTIATIONS = {
    # kind: (layout, optimizer, hyper-parameters, moving average, selection options)
    "sgd_single": ([(0, 33001)], "sgd", {}, None, None),
    "sgd_multi": (_WIDE_MULTI, "sgd", {}, None, None),
    "sgd_multi_clip": (_WIDE_MULTI, "sgd", dict(clip_norm=0.002), None, None),
    "momentum_single_clip_ema": ([(1, 33001)], "momentum", dict(clip_norm=0.002), 0.9, None),
    "rmsprop_single_ema": ([(0, 33001)], "rmsprop_mom", {}, 0.99, None),
    "rmsprop_multi_ema": (_WIDE_MULTI, "rmsprop_mom", {}, 0.9, None),
    "rmsprop_multi_clip": (_WIDE_MULTI, "rmsprop_mom", dict(clip_norm=0.002), None, None),
    "rmsprop_multi_clip_ema": (_WIDE_MULTI, "rmsprop_mom", dict(clip_norm=0.002), 0.9, None),
    "momentum_multi_ema": (_WIDE_MULTI, "momentum", {}, 0.9, None),
    "worker_clip_single": ([(0, 33001)], "momentum", dict(worker_clip_norm=1.8), None, None),
    "worker_clip_multi": (_WIDE_MULTI, "rmsprop_mom", dict(worker_clip_norm=2.2), None, None),
    "worker_clip_multi_then_clip": (_WIDE_MULTI, "sgd", dict(worker_clip_norm=2.2, clip_norm=0.002), 0.5, None),
    "worker_clip_single_deadline": ([(0, 33001)], "rmsprop_mom", dict(worker_clip_norm=1.8), None, "deadline"),
    "worker_clip_multi_deadline": (_WIDE_MULTI, "momentum", dict(worker_clip_norm=2.2), None, "deadline"),
    "sgd_multi_deadline_tags": (_WIDE_MULTI, "sgd", {}, None, "deadline+tags"),
}


@pytest.mark.parametrize("kind", sorted(_INSTANTIATIONS))
def test_every_compiled_launch_shape_every_instantiation_against_the_oracle(kind):
    import paper_1604_00981_amd as bs
    layout, opt, hyper, ema, sel_mode = _INSTANTIATIONS[kind]
    shapes = [bs.bsgd_get_shape(i) for i in range(bs.bsgd_num_shapes())]
    assert (256, 8, 2, 1) in shapes                     # the shape the timed workloads run in
    N, b = 21, 4
    results = []
    try:
        for shape in shapes:
            bs.bsgd_set_tuning(*shape)
            c = Case(N, b, layout, opt, seed=71, theta_shift=1, hyper=hyper, ema=ema)
            ranges = [(o, o + n) for o, n in layout]
            for step in range(2):
                g, t = c.draw(sigma=0.01)
                g *= c.r.uniform(0.2, 3.0, (c.W, 1)).astype(np.float32)
                covered = np.zeros(c.ld, bool)
                for lo, hi in ranges:
                    covered[lo:hi] = True
                g[:, ~covered] = 40.0                   # columns outside every tensor may not enter a norm or an update
                opts = None
                if sel_mode is not None:
                    opts = dict(deadline=float(np.sort(t)[N + 1 + step]), n_min=3)       # N+2, then N+3 messages in time
                    if "tags" in sel_mode:
                        opts.update(tags=np.where(c.r.random(c.W) < 0.2, step - 1, step).astype(np.int32), step_tag=step)
                if "worker_clip_norm" in hyper:
                    kept = (orc.select_first_n(t, N, b) if opts is None else
                            orc.select_ex(t, N, b, opts.get("tags"), opts.get("step_tag", 0), opts["deadline"], 3))[0]
                    sc = orc.worker_clip_scales(g, kept, ranges, c.hy["worker_clip_norm"])
                    assert (sc < 1).any() and (sc == 1).any()
                assert c.both(g, t, opts) == 0
                if sel_mode == "deadline":
                    assert bs.bsgd_last_kept_count(c.ws) == N + 2 + step
                if "clip_norm" in hyper:
                    assert bs.bsgd_last_clip(c.ws)[1] < 1.0                              # the clip of the mean is active
            c.compare()
            results.append(c.gpu_arrays())
    finally:
        bs.bsgd_set_tuning()
    if "clip_norm" not in hyper and "worker_clip_norm" not in hyper:
        for a, bb in zip(results, results[1:]):
            for k in a:
                assert np.array_equal(a[k], bb[k]), k   # rows are added in the same order whatever the shape


_FUSED_KINDS = {
    # kind: (N, b, layout, optimizer, hyper-parameters, moving average, selection options)
    "sgd_single": (4, 1, [(0, 70_001)], "sgd", {}, None, None),
    "rmsprop_multi_ema": (9, 3, [(3, 9001), (9004, 17), (9100, 20000)], "rmsprop_mom", {}, 0.9, None),
    "momentum_multi_clip": (9, 3, [(3, 9001), (9004, 17), (9100, 20000)], "momentum", dict(clip_norm=0.003), None, None),
    "sgd_clip_ema_64_workers": (60, 4, [(1, 30_011)], "sgd", dict(clip_norm=0.001), 0.5, None),
    "momentum_deadline_tags": (7, 4, [(0, 12_345), (12_345, 678)], "momentum", {}, None, "deadline+tags"),
}


@pytest.mark.parametrize("kind", sorted(_FUSED_KINDS))
def test_selection_inside_the_step_launch_equals_the_separate_kernel(kind):
    # A step's first launch ranks the arrival times itself (every wavefront, from a 64-bit mask of the kept rows);
    # with that switched off the same step runs k_select first.  Same bits, same recorded outputs;
    # both against the oracle.  Then too few arrivals: nothing may be touched either way.
    import paper_1604_00981_amd as bs
    N, b, layout, opt, hyper, ema, sel_mode = _FUSED_KINDS[kind]
    out = {}
    try:
        for fused in (True, False):
            bs.bsgd_set_fused_selection(fused)
            c = Case(N, b, layout, opt, seed=95, theta_shift=1, hyper=hyper, ema=ema)
            rec = []
            for step in range(3):
                g, t = c.draw()
                opts = None
                if sel_mode is not None:
                    opts = dict(deadline=float(np.sort(t)[N + step]), n_min=3, step_tag=step,
                                tags=np.where(c.r.random(c.W) < 0.2, step - 1, step).astype(np.int32))
                assert c.both(g, t, opts) == 0
                assert bs.bsgd_last_step_fused_selection() == fused
                assert bs.bsgd_last_launch_count() == (2 if "clip_norm" in hyper else 1)
                nk = bs.bsgd_last_kept_count(c.ws)
                rec.append((nk, bs.bsgd_last_selection(c.ws, nk), bs.bsgd_last_status(c.ws), bs.bsgd_last_gradient_count(c.ws)))
            c.compare()
            before = c.gpu_arrays()
            g, t = c.draw()
            t[:b + 1] = np.inf                                   # one arrival short
            assert c.both(g, t, None if sel_mode is None else dict(n_min=N)) == bs.BSGD_ERR_TOO_FEW
            assert bs.bsgd_last_step_fused_selection() == fused
            assert bs.bsgd_last_kept_count(c.ws) == 0
            after = c.gpu_arrays()
            for k in before:
                assert np.array_equal(before[k], after[k]), k
            out[fused] = (after, rec)
    finally:
        bs.bsgd_set_fused_selection(True)
    assert out[True][1] == out[False][1]
    for k in out[True][0]:
        assert np.array_equal(out[True][0][k], out[False][0][k]), k


def test_where_the_selection_runs():
    import paper_1604_00981_amd as bs
    # more than 64 workers: a kernel of its own
    c = Case(70, 5, [(0, 3001)], "sgd", seed=96)
    c.both(*c.draw())
    assert not bs.bsgd_last_step_fused_selection()
    # per-worker clipping needs the kept rows before its norm pass: a kernel of its own
    c = Case(5, 2, [(0, 3001)], "sgd", seed=97, hyper=dict(worker_clip_norm=0.5))
    c.both(*c.draw())
    assert not bs.bsgd_last_step_fused_selection()
    # tensors far apart: two runs of chunks, two launches; the first does the selection, the second reads what it published
    c = Case(5, 2, [(0, 3001), (1_200_000, 3001)], "sgd", seed=98)
    for _ in range(2):
        c.both(*c.draw())
    assert bs.bsgd_last_step_fused_selection() and bs.bsgd_last_launch_count() == 2
    c.compare()
    # many rows over many columns: several rounds; again only the first launch ranks the arrival times
    c = Case(40, 2, [(0, 5_400_000)], "rmsprop_mom", seed=99)
    for _ in range(2):
        c.both(*c.draw())
    assert bs.bsgd_last_step_fused_selection() and bs.bsgd_last_launch_count() >= 2
    c.compare()
    # ... and when too few arrive, no launch of the step touches anything
    before = c.gpu_arrays()
    g, t = c.draw()
    t[:3] = np.inf
    assert c.both(g, t) == bs.BSGD_ERR_TOO_FEW
    after = c.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    # the same large step with the selection as a kernel of its own: the same bits
    try:
        bs.bsgd_set_fused_selection(False)
        d = Case(40, 2, [(0, 5_400_000)], "rmsprop_mom", seed=99)
        for _ in range(2):
            d.both(*d.draw())
        assert not bs.bsgd_last_step_fused_selection()
    finally:
        bs.bsgd_set_fused_selection(True)
    gd = d.gpu_arrays()
    for k in before:
        assert np.array_equal(before[k], gd[k]), k


@pytest.mark.parametrize("seed", range(48))
def test_random_configurations_against_the_oracle(seed):
    # every option drawn at random and combined freely: optimizer, clip of the mean, per-worker clip, moving average,
    # tags, deadline mode, number of workers (up to 256), layout (single or many tensors, gaps, unaligned starts,
    # misaligned allocations), row stride padding, launch shape (automatic or any compiled one)
    import paper_1604_00981_amd as bs
    r = np.random.default_rng(1000 + seed)
    W = int(r.choice([2, 5, 9, 33, 64, 65, 130, 256]))
    N = int(r.integers(1, W + 1))
    b = W - N
    opt = str(r.choice(["sgd", "momentum", "rmsprop_mom"]))
    T = int(r.choice([1, 1, 2, 7, 40]))
    total = int(r.choice([700, 9_000, 70_000]) if W > 64 else r.choice([700, 9_000, 70_000, 400_000]))
    cuts = np.sort(r.choice(np.arange(1, total), T - 1, replace=False)) if T > 1 else np.array([], int)
    sizes = [int(x) for x in np.diff(np.concatenate([[0], cuts, [total]]))]
    layout, o = [], int(r.integers(0, 7))
    for n in sizes:
        layout.append((o, n))
        o += n + (int(r.integers(1, 3000)) if r.random() < 0.3 else 0)
    span = layout[-1][0] + layout[-1][1]
    hyper = {}
    sigma = 0.01
    if r.random() < 0.4:
        hyper["clip_norm"] = float(sigma * np.sqrt(sum(sizes) / N) * r.uniform(0.3, 1.5))      # around the norm of the mean
    if r.random() < 0.35:
        hyper["worker_clip_norm"] = float(sigma * np.sqrt(sum(sizes)) * r.uniform(0.6, 1.6))   # around a row's norm
    ema = float(r.choice([0.0, 0.5, 0.9999])) if r.random() < 0.4 else None
    ld = (span + 3) // 4 * 4 + 4 * int(r.integers(0, 5))
    shapes = [None] + [bs.bsgd_get_shape(i) for i in range(bs.bsgd_num_shapes())]
    shape = shapes[int(r.integers(0, len(shapes)))]
    use_tags, use_deadline = r.random() < 0.3, r.random() < 0.3
    try:
        if shape is not None:
            bs.bsgd_set_tuning(*shape)
        c = Case(N, b, layout, opt, seed=2000 + seed, ld=ld, theta_shift=int(r.integers(0, 4)), hyper=hyper, ema=ema)
        done = 0
        for step in range(3):
            g, t = c.draw(sigma=sigma)
            g *= c.r.uniform(0.5, 2.0, (c.W, 1)).astype(np.float32)
            opts = None
            if use_tags or use_deadline:
                opts = {}
                if use_tags:
                    opts.update(tags=np.where(c.r.random(W) < 0.15, step - 1, step).astype(np.int32), step_tag=step)
                if use_deadline:
                    opts.update(deadline=float(np.sort(t)[int(c.r.integers(0, W))]), n_min=int(c.r.integers(1, N + 1)))
            status = c.both(g, t, opts)                 # kept set, t_step, status and kept count against the oracle
            assert status in (0, bs.BSGD_ERR_TOO_FEW)
            done += status == 0
        if done:
            c.compare()
    finally:
        bs.bsgd_set_tuning()


def _irregular_layout(total, count, seed, crowded=0):
    """`count` tensors of irregular sizes packed back to back over about `total` columns; with `crowded`, that many
    tiny tensors come first (more than one launch can carry as an argument)."""
    r = np.random.default_rng(seed)
    sizes = [int(x) for x in r.integers(1, 90, crowded)]
    cuts = np.sort(r.choice(np.arange(1, total), count - 1, replace=False))
    sizes += [int(x) for x in np.diff(np.concatenate([[0], cuts, [total]]))]
    layout, o = [], 3                                   # the first tensor does not start on a 16-byte group
    for n in sizes:
        layout.append((o, n))
        o += n
    return layout


@pytest.mark.parametrize("N", [12, 3])
@pytest.mark.parametrize("crowded", [0, 200])
@pytest.mark.parametrize("clip", [0.0, 0.004])
def test_tensor_table_as_argument_or_through_workspace_same_bits(crowded, clip, N):
    # 11 M columns in the widest shape go out as three launches; each launch sees its own window of the table.
    # crowded = 0: every window fits the argument buffer; crowded = 200: the first window does not, so the call
    # writes the table into the workspace.  Forcing the workspace path must not change a bit.  With N = 3 kept rows,
    # and in the clipped variants, 1.4 M columns go out as one launch per pass, whose window holds every segment.
    import paper_1604_00981_amd as bs
    layout = _irregular_layout(11_000_000 if (N > 8 and clip == 0.0) else 1_400_000, 120, seed=31, crowded=crowded)
    results, launches = [], []
    try:
        bs.bsgd_set_tuning(256, 8, 2, 1)
        for mode in (0, 1):
            bs.bsgd_set_table_mode(mode)
            c = Case(N, 1, layout, "rmsprop_mom", seed=32, hyper=dict(clip_norm=clip))
            for _ in range(2):
                c.both(*c.draw())
            c.compare()
            launches.append(bs.bsgd_last_launch_count())
            results.append(c.gpu_arrays())
    finally:
        bs.bsgd_set_table_mode(0)
        bs.bsgd_set_tuning()
    if clip == 0.0:
        assert launches[0] == (3 if N > 8 else 1)       # three launches: the windows differ from launch to launch
    for k in results[0]:
        assert np.array_equal(results[0][k], results[1][k]), k


def test_async_server_case_N1_b0():
    # Algorithm 2's server: apply the one gradient that arrived
    c = Case(1, 0, [(0, 1030)], "sgd", seed=19)
    g, t = c.draw()
    th0 = c.gpu_arrays()["theta"]
    c.gpu_step(g, t)
    ref = th0 - np.float32(c.hy["lr"]) * g[0, :1030]
    np.testing.assert_allclose(c.gpu_arrays()["theta"], ref, rtol=1e-6, atol=1e-9)


def test_max_workers():
    c = Case(250, 6, [(0, 2051)], "momentum", seed=20)
    c.both(*c.draw())
    c.compare()


def test_maximum_number_of_tensors():
    # 4096 tensors (the documented maximum), tiny and odd-sized, a gap after every third one:
    # the segment table (tensors and gaps) fills the whole LDS staging area of the multi-tensor path
    import paper_1604_00981_amd as bs
    r = np.random.default_rng(77)
    layout, o = [], 2
    for j in range(bs.BSGD_MAX_TENSORS):
        n = int(r.integers(1, 60))
        layout.append((o, n))
        o += n + (int(r.integers(1, 9)) if j % 3 == 2 else 0)
    c = Case(5, 2, layout, "momentum", seed=78, ema=0.9)
    for _ in range(2):
        c.both(*c.draw())
    c.compare()
    cc = Case(5, 2, layout, "rmsprop_mom", seed=79, hyper=dict(clip_norm=0.05, worker_clip_norm=0.4))
    cc.both(*cc.draw())
    cc.compare()
