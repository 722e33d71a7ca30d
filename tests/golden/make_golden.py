#!/usr/bin/env python3
"""Writes tests/golden/kept_sets.json: for every workload configuration and
step, the arrival times (as fp32 bit patterns) and the kept worker set.

The paper prints no worked numeric example of a step, so there are no paper
values to store.  These fixtures are regression anchors: they are produced by
calling ONLY the seeded workload generator and the CPU oracle (Algorithm 4's
collect loop: first N of N+b arrivals), never the GPU path.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl                       # noqa: E402
from oracle import bsgd_oracle as orc        # noqa: E402


def main() -> None:
    out = {}
    for name in ("C1", "C2", "C3", "C4", "C5"):
        cfg = wl.get_config(name)
        steps = []
        for step in range(cfg.steps):
            t = wl.arrival_times(cfg, step)
            sel, t_step = orc.select_first_n(t, cfg.N, cfg.b)
            steps.append({"arrival_bits": [int(x) for x in t.view(np.uint32)],
                          "kept": [int(k) for k in sel],
                          "t_step_bits": int(np.float32(t_step).view(np.uint32))})
        out[name] = {"N": cfg.N, "b": cfg.b, "seed": cfg.seed, "steps": steps}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "kept_sets.json")
    with open(path, "w") as f:
        json.dump(out, f, separators=(",", ":"))
    print("wrote", path)


if __name__ == "__main__":
    main()
