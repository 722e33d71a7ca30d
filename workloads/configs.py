"""The five step configurations (C1..C5) the build is measured and tested on.

Shapes follow the paper's workloads: 50-100 kept workers with a handful of
backups (Sec. 3.1 and Sec. 4 use N in {50..100}, b in {0,1,4,6}), RMSProp
with momentum at decay 0.9 / momentum 0.9 (Appendix A.2/A.3), and arrival
times with a long right tail (Sec. 3.1, Figures 3-4).  Model sizes,
distributions and seeds are this build's synthetic stand-ins.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class StepConfig:
    name: str
    seed: int
    steps: int
    N: int                      # gradients kept per step
    b: int                      # backup workers
    P: int                      # total fp32 parameters (target total for 'loguniform')
    T: int                      # number of parameter tensors
    tensor_mode: str            # 'flat' | 'equal' | 'loguniform'
    theta_sigma: float
    grad_sigma: float
    worker_scale: Optional[Tuple[float, float]]   # U(lo,hi) multiplier per worker
    tensor_scale: Optional[Tuple[float, float]]   # U(lo,hi) multiplier per tensor
    arrival: str                # 'shifted_exp' | 'lognormal'
    arrival_shift: float = 0.0
    arrival_rate: float = 1.0
    arrival_sigma: float = 0.0
    straggler_p: float = 0.0
    straggler_lo: float = 2.0
    straggler_hi: float = 10.0
    opt: str = "sgd"            # 'sgd' | 'momentum' | 'rmsprop_mom'
    lr: float = 0.1
    momentum: float = 0.0
    decay: float = 0.0
    eps: float = 0.0
    clip_norm: float = 0.0      # <= 0: clipping off
    warmup_steps: int = 0       # linear warm-up of the learning rate
    tensor_min: int = 64
    tensor_max: int = 2_000_000

    @property
    def W(self) -> int:
        return self.N + self.b


CONFIGS = {
    "C1": StepConfig(
        name="C1", seed=0, steps=10, N=4, b=1, P=1_048_576, T=1, tensor_mode="flat",
        theta_sigma=0.05, grad_sigma=0.01, worker_scale=None, tensor_scale=None,
        arrival="shifted_exp", arrival_shift=1.0, arrival_rate=1.0,
        opt="sgd", lr=0.1),
    "C2": StepConfig(
        name="C2", seed=1, steps=20, N=50, b=4, P=25_000_000, T=1, tensor_mode="flat",
        theta_sigma=0.02, grad_sigma=1e-3, worker_scale=(0.5, 1.5), tensor_scale=None,
        arrival="lognormal", arrival_sigma=0.25, straggler_p=0.05,
        opt="rmsprop_mom", lr=0.045, momentum=0.9, decay=0.9, eps=1.0),
    "C3": StepConfig(
        name="C3", seed=2, steps=20, N=100, b=6, P=25_000_000, T=1, tensor_mode="flat",
        theta_sigma=0.02, grad_sigma=1e-3, worker_scale=None, tensor_scale=None,
        arrival="lognormal", arrival_sigma=0.4,
        opt="momentum", lr=0.1, momentum=0.9, warmup_steps=5),
    "C4": StepConfig(
        name="C4", seed=3, steps=10, N=50, b=2, P=24_000_000, T=300, tensor_mode="loguniform",
        theta_sigma=0.02, grad_sigma=1e-3, worker_scale=None, tensor_scale=(0.1, 10.0),
        arrival="shifted_exp", arrival_shift=1.0, arrival_rate=2.0,
        opt="rmsprop_mom", lr=0.045, momentum=0.9, decay=0.9, eps=1.0),
    "C5": StepConfig(
        name="C5", seed=4, steps=5, N=32, b=2, P=134_217_728, T=64, tensor_mode="equal",
        theta_sigma=0.02, grad_sigma=1e-3, worker_scale=None, tensor_scale=None,
        arrival="lognormal", arrival_sigma=0.3,
        opt="momentum", lr=0.05, momentum=0.9, clip_norm=1.0),
}


def get_config(name: str) -> StepConfig:
    return CONFIGS[name]


def scaled_config(name: str, P: int, **overrides) -> StepConfig:
    """The named configuration with a smaller parameter count (same N, b,
    optimizer, distributions and seed), for cases the CPU oracle must finish
    in seconds."""
    cfg = CONFIGS[name]
    kw = dict(P=P, name=f"{cfg.name}@P={P}")
    if cfg.tensor_mode == "loguniform":
        # keep the size spread: shrink the upper bound with the total
        kw["tensor_max"] = max(cfg.tensor_min * 4, int(cfg.tensor_max * P / cfg.P))
    kw.update(overrides)
    return replace(cfg, **kw)
