"""The stored kept sets (written by tests/golden/make_golden.py from the
oracle alone) still match what the generator and the oracle produce, and the
GPU selection reproduces them bit for bit."""
import json
import os

import numpy as np
import pytest

import workloads as wl
from oracle import bsgd_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "kept_sets.json")


def _load():
    with open(GOLDEN) as f:
        return json.load(f)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_generator_and_oracle_reproduce_the_fixture(name):
    g = _load()[name]
    cfg = wl.get_config(name)
    assert (g["N"], g["b"], g["seed"], len(g["steps"])) == (cfg.N, cfg.b, cfg.seed, cfg.steps)
    for step, rec in enumerate(g["steps"]):
        t = wl.arrival_times(cfg, step)
        assert [int(x) for x in t.view(np.uint32)] == rec["arrival_bits"]
        sel, t_step = orc.select_first_n(t, cfg.N, cfg.b)
        assert sel.tolist() == rec["kept"]
        assert int(np.float32(t_step).view(np.uint32)) == rec["t_step_bits"]
        # the fixture itself obeys the definition: every kept arrival precedes every dropped one
        kept = set(rec["kept"])
        worst_kept = max((float(t[k]), k) for k in kept)
        dropped = [(float(t[k]), k) for k in range(cfg.W) if k not in kept]
        assert all(worst_kept < d for d in dropped)


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_gpu_selection_reproduces_the_fixture(name):
    import torch
    import paper_1604_00981_amd as bs
    g = _load()[name]
    N, b = g["N"], g["b"]
    for rec in g["steps"]:
        t = np.array(rec["arrival_bits"], dtype=np.uint32).view(np.float32)
        sel = torch.zeros(N, dtype=torch.int32, device="cuda")
        ts = torch.zeros(1, dtype=torch.float32, device="cuda")
        st = torch.zeros(1, dtype=torch.int32, device="cuda")
        bs.bsgd_select_first_n(torch.from_numpy(t).cuda(), N, b, sel, ts, st)
        torch.cuda.synchronize()
        assert st.item() == 0
        assert sel.cpu().tolist() == rec["kept"]
        assert int(ts.cpu().numpy().view(np.uint32)[0]) == rec["t_step_bits"]
