"""Seeded synthetic inputs for the pod-rollout hot path.

This module only *draws numbers*: market paths, technical indicators, action
noise and network weights, in the shapes of the paper's stock-trading workload
(Table 1: balance, shares, close prices, technical indicators; Fig. 6: initial
capital 1e6).  The paper's own market data (minute-level NASDAQ-100 from a
licensed database, Sec. 5.3) is not available, so geometric-Brownian-motion
paths stand in for it.

None of the method's arithmetic (observation assembly, MLP, trading rules,
GAE) lives here; both the HIP path and the CPU checker consume these tensors.

Streams (numpy SeedSequence spawn keys, base seed 211205923):
    0 = initial prices, 1 = GBM shocks, 2 = indicators, 3 = action noise,
    4 = actor weights, 5 = critic weights (then one key per agent).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

BASE_SEED = 211205923


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and constants of one rollout workload."""

    name: str
    index: int            # position in the list of named workloads (seed key)
    n_envs: int           # N
    n_agents: int         # P, N % P == 0
    n_stocks: int         # D
    n_ind: int            # K indicators per stock
    hidden: int           # width of both hidden layers
    steps: int            # T rollout steps (episode horizon H = T by default)
    mlp_dtype: int        # 0 = fp32 operands, 1 = bf16 operands + fp32 accumulate
    gbm_sigma: float      # per-step volatility of the price paths
    cash0: float = 1.0e6
    hmax: float = 100.0
    cost: float = 1.0e-3
    sigma: float = 0.5
    gamma: float = 0.99
    lam: float = 0.95
    reward_scale: float = 2.0 ** -12
    obs_scale: tuple = (2.0 ** -20, 2.0 ** -7, 2.0 ** -10, 1.0)

    @property
    def state_dim(self) -> int:
        return 1 + 2 * self.n_stocks + self.n_stocks * self.n_ind

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny", 0, 16, 1, 5, 2, 64, 64, 0, 0.02),
        Workload("dow30", 1, 4096, 1, 30, 8, 256, 1024, 0, 0.015),
        Workload("large", 2, 16384, 1, 30, 8, 512, 1024, 1, 0.015),
        Workload("wide", 3, 2048, 1, 500, 4, 1024, 512, 1, 0.015),
        Workload("tournament", 4, 65536, 64, 30, 8, 256, 512, 0, 0.015),
    ]
}


def _rng(w: Workload, stream: int, agent: Optional[int] = None) -> np.random.Generator:
    key = (w.index, stream) if agent is None else (w.index, stream, agent)
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(BASE_SEED, spawn_key=key)))


def make_market(w: Workload, horizon: Optional[int] = None, n_market: Optional[int] = None):
    """Price paths [H+1, M, D] and indicators [H+1, M, D*K], float32.

    p0 ~ U[10, 100]; log-returns are -s^2/2 + s*z with z ~ N(0,1) (zero drift
    of the price itself); computed in float64 and cast once.  Indicators are
    i.i.d. N(0,1), independent of prices.
    """
    H = w.steps if horizon is None else horizon
    M = w.n_envs if n_market is None else n_market
    D, K = w.n_stocks, w.n_ind
    p0 = _rng(w, 0).uniform(10.0, 100.0, size=(M, D))
    z = _rng(w, 1).standard_normal(size=(H, M, D))
    s = w.gbm_sigma
    logp = np.empty((H + 1, M, D), dtype=np.float64)
    logp[0] = np.log(p0)
    np.cumsum(-0.5 * s * s + s * z, axis=0, out=z)
    logp[1:] = logp[0][None] + z
    price = np.exp(logp).astype(np.float32)
    ind = _rng(w, 2).standard_normal(size=(H + 1, M, D * K), dtype=np.float32)
    return price, ind


def make_noise(w: Workload, steps: Optional[int] = None) -> np.ndarray:
    """Action noise eps ~ N(0,1), float32 [T, N, D]."""
    T = w.steps if steps is None else steps
    return _rng(w, 3).standard_normal(size=(T, w.n_envs, w.n_stocks), dtype=np.float32)


def make_weights(w: Workload, critic: bool):
    """Weights and biases ~ N(0, 0.1^2), float32.

    Returns dict W1 [P,S,Hd], b1 [P,Hd], W2 [P,Hd,Hd], b2 [P,Hd], W3 [P,Hd,O],
    b3 [P,O] with O = D (actor) or 1 (critic); one independent draw per agent.
    """
    S, Hd = w.state_dim, w.hidden
    O = 1 if critic else w.n_stocks
    shapes = {"W1": (S, Hd), "b1": (Hd,), "W2": (Hd, Hd), "b2": (Hd,), "W3": (Hd, O), "b3": (O,)}
    out = {k: np.empty((w.n_agents,) + s, dtype=np.float32) for k, s in shapes.items()}
    for g in range(w.n_agents):
        r = _rng(w, 5 if critic else 4, g)
        for k, s in shapes.items():
            out[k][g] = (0.1 * r.standard_normal(size=s)).astype(np.float32)
    return out


def make_all(w: Workload, horizon: Optional[int] = None, n_market: Optional[int] = None,
             steps: Optional[int] = None):
    """Host-side bundle of every input of one workload (numpy, bit-portable)."""
    price, ind = make_market(w, horizon, n_market)
    return {
        "price": price,
        "ind": ind,
        "noise": make_noise(w, steps),
        "actor": make_weights(w, critic=False),
        "critic": make_weights(w, critic=True),
    }


def make_all_device(w: Workload, device, horizon: Optional[int] = None,
                    n_market: Optional[int] = None, steps: Optional[int] = None):
    """Same recipe drawn on an accelerator with a seeded torch.Generator.

    For workloads whose tensors are tens of GB (the host generator would need
    minutes and more RAM than the tensors themselves).  The draws differ from
    the numpy ones; parity tests copy the slices they check back to the host,
    so both sides still see identical bytes.  Weights stay on the numpy recipe.
    """
    import torch

    H = w.steps if horizon is None else horizon
    M = w.n_envs if n_market is None else n_market
    T = w.steps if steps is None else steps
    D, K, N = w.n_stocks, w.n_ind, w.n_envs
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED * 8 + w.index)
    s = w.gbm_sigma
    logp = torch.empty((H + 1, M, D), dtype=torch.float64, device=device)
    logp[0] = torch.log(10.0 + 90.0 * torch.rand((M, D), generator=g, dtype=torch.float64, device=device))
    # row-chunked so the float64 temporaries stay small next to the outputs
    step_rows = max(1, (1 << 26) // max(1, M * D))
    for r0 in range(0, H, step_rows):
        r1 = min(H, r0 + step_rows)
        z = torch.randn((r1 - r0, M, D), generator=g, dtype=torch.float64, device=device)
        z.mul_(s).add_(-0.5 * s * s)
        torch.cumsum(z, dim=0, out=z)
        logp[r0 + 1:r1 + 1] = logp[r0][None] + z
        del z
    price = torch.exp(logp).to(torch.float32)
    del logp
    ind = torch.empty((H + 1, M, D * K), dtype=torch.float32, device=device)
    ind.normal_(generator=g)
    noise = torch.empty((T, N, D), dtype=torch.float32, device=device)
    noise.normal_(generator=g)
    to_dev = lambda d: {k: torch.from_numpy(v).to(device) for k, v in d.items()}
    return {
        "price": price,
        "ind": ind,
        "noise": noise,
        "actor": to_dev(make_weights(w, critic=False)),
        "critic": to_dev(make_weights(w, critic=True)),
    }


def bytes_per_env_step(w: Workload) -> int:
    """Algorithmic HBM bytes of one env-step with persistent state.

    Reads: noise 4D + next market row 4D(1+K); writes: observation 4S, raw
    action 4D, reward 4 + done 1 + log-prob 4 (rounded up to 12)."""
    D, K = w.n_stocks, w.n_ind
    return 20 * D + 8 * D * K + 16


def mlp_flops_per_env_step(w: Workload, critic: bool) -> int:
    S, Hd = w.state_dim, w.hidden
    O = 1 if critic else w.n_stocks
    return 2 * (S * Hd + Hd * Hd + Hd * O)
