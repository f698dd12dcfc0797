"""The five synthetic configurations (inputs only, shared by the harness and by the oracle's tests).

They stand in for the paper's ResNet-18 / ResNet-50 runs on CIFAR-10 / ImageNet with up to 64 workers on ring,
exponential and complete graphs (section "Numerical Experiments"): same flat-vector sizes, worker counts,
topologies and communication rates, with Gaussian initial parameters and an affine-plus-noise gradient model in
place of datasets and networks.  Nothing here performs any of the method's arithmetic.
"""
from dataclasses import dataclass, field, replace

import numpy as np

from . import gen

GAMMA = 0.1   # base learning rate of the paper's experiments ("Hyper-parameters" paragraph)


@dataclass(frozen=True)
class Config:
    name: str
    n: int
    topology: str            # complete | ring | exponential
    d: int
    init_sigma: float
    gscale: float            # s of g = s (x - c_i) + xi
    use_c: bool
    xi_sigma: float          # 0: no noise buffer
    edge_rate: float         # per edge; for straggler configs a multiple of the mean node rate
    events: int
    seed: int
    straggler_sigma: float = 0.0     # > 0: node rates ~ LogNormal(0, sigma), edge rate = edge_rate * mean
    accelerated: bool = True         # Proposition 3.2 accelerated setting; False: eta = 0 baseline
    eta: float = None                # explicit override (config 1 fixes eta = 0.5)
    alpha_tilde: float = None        # explicit override
    gamma: float = GAMMA
    curvature: bool = False          # per-worker, per-coordinate curvatures h_i (strongly convex local quadratics)
    extra: dict = field(default_factory=dict)


CONFIGS = {
    "C1": Config("C1", 4, "complete", 1_000, 1.0, 1.0, True, 0.0, 1.0, 10_000, 0xA2C1D2 + 1, eta=0.5),
    "C2": Config("C2", 16, "ring", 1_000_000, 1.0, 1.0, True, 0.1, 1.0, 100_000, 0xA2C1D2 + 2),
    "C3": Config("C3", 64, "ring", 11_700_000, 0.01, 0.0, False, 1e-3, 2.0, 1_000_000, 0xA2C1D2 + 3),
    "C4": Config("C4", 64, "exponential", 25_600_000, 0.01, 0.0, False, 1e-3, 1.0, 1_000_000, 0xA2C1D2 + 4),
    "C4-baseline": Config("C4-baseline", 64, "exponential", 25_600_000, 0.01, 0.0, False, 1e-3, 1.0, 1_000_000,
                          0xA2C1D2 + 4, accelerated=False, alpha_tilde=0.0),
    "C5": Config("C5", 64, "complete", 25_600_000, 1.0, 1.0, True, 0.1, 0.5, 2_000_000, 0xA2C1D2 + 5,
                 straggler_sigma=0.5),
}

DOMAIN_RATE = 4    # generator domain for the straggler node rates (row 0, column = worker)


def clock_rates(cfg):
    """(node_rate[n], edge_rate scalar) of a config."""
    if cfg.straggler_sigma > 0:
        z = gen.normal(cfg.seed, DOMAIN_RATE, 0, np.arange(cfg.n)).astype(np.float64)
        node = np.exp(cfg.straggler_sigma * z)
        return node, cfg.edge_rate * float(node.mean())
    return np.ones(cfg.n), float(cfg.edge_rate)


def scaled(cfg, d=None, events=None):
    """Same workload at another d / event count (parity tests, CPU-baseline samples)."""
    return replace(cfg, d=cfg.d if d is None else int(d), events=cfg.events if events is None else int(events))
