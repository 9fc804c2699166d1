"""Thin ctypes binding of libpodrollout.so (include/podrollout.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
the library.  torch supplies device memory and the current HIP stream.  There
is no CPU fallback: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpodrollout.so")

PR_OK, PR_EINVAL, PR_ENOMEM, PR_EHIP, PR_EUNSUPPORTED, PR_ETOOBIG = 0, -1, -2, -3, -4, -5
PR_STATIC_SCRATCH_BYTES = 24 << 20
PR_MLP_F32, PR_MLP_BF16 = 0, 1
PR_SCHED_STEPWISE, PR_SCHED_FUSED = 0, 1
PR_NET_ACTOR, PR_NET_CRITIC = 0, 1

EXPORTS = ["rollout_workspace_bytes", "rollout_kernel_lds_bytes", "rollout_init", "rollout_set_weights", "rollout_reset", "rollout_set_replay",
           "rollout_step_T",
           "rollout_step_forced", "rollout_mlp_forward", "rollout_get_state", "rollout_set_state", "compute_gae",
           "trading_metrics", "population_refill", "ppo_workspace_bytes",
           "ppo_minibatch_grads", "ppo_minibatch_grads_noalloc", "adam_update", "ppo_learner_step", "rollout_leaderboard", "rollout_calibrate",
           "rollout_destroy", "rollout_strerror", "rollout_last_hip_error"]


class PrPpoConfig(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_stocks", C.c_int32), ("n_ind", C.c_int32), ("hidden", C.c_int32),
                ("sigma", C.c_float), ("clip", C.c_float), ("value_coef", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float), ("adam_step", C.c_int32)]


class PrNetParams(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]


class PrConfig(C.Structure):
    _fields_ = [("n_envs", C.c_int32), ("n_agents", C.c_int32), ("n_stocks", C.c_int32), ("n_ind", C.c_int32),
                ("hidden", C.c_int32), ("horizon", C.c_int32), ("n_market", C.c_int32), ("mlp_dtype", C.c_int32),
                ("schedule", C.c_int32), ("cash0", C.c_float), ("hmax", C.c_float), ("cost", C.c_float),
                ("sigma", C.c_float), ("reward_scale", C.c_float), ("obs_scale", C.c_float * 4)]


class PrMarket(C.Structure):
    _fields_ = [("price", C.c_void_p), ("ind", C.c_void_p)]


class PrWeights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]


class PrBuffers(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("obs", "act_raw", "reward", "done", "value", "logp", "mu", "shares")]


class PrState(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("cash", "holdings", "cursor", "ep_return", "ep_sum", "ep_sqsum",
                                          "ep_count")]


class PodError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().rollout_strerror(code).decode()
        if code == PR_EHIP:
            msg += f" (hipError {lib().rollout_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


_lib = None


def lib():
    """Load the HIP library; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2112_05923_amd.build` "
                "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        l.rollout_strerror.restype = C.c_char_p
        l.rollout_strerror.argtypes = [C.c_int]
        l.rollout_workspace_bytes.argtypes = [C.POINTER(PrConfig), C.POINTER(C.c_size_t)]
        l.rollout_kernel_lds_bytes.argtypes = [C.POINTER(PrConfig), C.c_int32, C.POINTER(C.c_size_t)]
        l.rollout_init.argtypes = [C.POINTER(PrConfig), C.POINTER(PrMarket), C.POINTER(PrWeights),
                                   C.POINTER(PrWeights), C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
        l.rollout_set_weights.argtypes = [C.c_void_p, C.POINTER(PrWeights), C.POINTER(PrWeights)]
        l.rollout_reset.argtypes = [C.c_void_p]
        l.rollout_set_replay.argtypes = [C.c_void_p, C.POINTER(PrMarket), C.c_int32, C.c_void_p]
        l.rollout_step_T.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(PrBuffers)]
        l.rollout_step_forced.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(PrBuffers)]
        l.rollout_mlp_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        l.rollout_get_state.argtypes = [C.c_void_p, C.POINTER(PrState)]
        l.rollout_set_state.argtypes = [C.c_void_p, C.POINTER(PrState)]
        l.compute_gae.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                  C.c_float, C.c_void_p, C.c_void_p]
        l.trading_metrics.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_float), C.c_double, C.c_double, C.c_void_p, C.c_void_p]
        l.population_refill.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_int32, C.c_float, C.c_void_p,
                                        C.c_void_p]
        NP = C.POINTER(PrNetParams)
        l.ppo_workspace_bytes.argtypes = [C.POINTER(PrPpoConfig), C.POINTER(C.c_size_t)]
        l.ppo_minibatch_grads.argtypes = [C.c_void_p, C.POINTER(PrPpoConfig)] + [C.c_void_p] * 6 + [NP] * 4 + [
            C.c_void_p, C.c_size_t, C.c_void_p]
        l.ppo_minibatch_grads_noalloc.argtypes = [C.c_void_p, C.POINTER(PrPpoConfig)] + [C.c_void_p] * 6 + [NP] * 4 + [
            C.c_void_p]
        l.adam_update.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                  C.c_float, C.c_float, C.c_float, C.c_int32]
        l.ppo_learner_step.argtypes = [C.c_void_p, C.POINTER(PrPpoConfig)] + [C.c_void_p] * 6 + [NP] * 6 + [
            C.c_void_p, C.c_size_t, C.c_void_p]
        l.rollout_leaderboard.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.rollout_calibrate.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]
        l.rollout_destroy.argtypes = [C.c_void_p]
        _lib = l
    return _lib


def _check(code: int, where: str):
    if code != PR_OK:
        raise PodError(code, where)


def _dev(t: torch.Tensor, dtype, shape=None, name="tensor"):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous cuda tensor of {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != {tuple(shape)}")
    return t.data_ptr()


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_config(w, horizon: Optional[int] = None, n_market: Optional[int] = None,
                schedule: int = PR_SCHED_STEPWISE) -> PrConfig:
    """pr_config from any object with the workload's field names."""
    c = PrConfig()
    c.n_envs, c.n_agents, c.n_stocks, c.n_ind = w.n_envs, w.n_agents, w.n_stocks, w.n_ind
    c.hidden = w.hidden
    c.horizon = w.steps if horizon is None else horizon
    c.n_market = w.n_envs if n_market is None else n_market
    c.mlp_dtype = w.mlp_dtype
    c.schedule = schedule
    c.cash0, c.hmax, c.cost, c.sigma, c.reward_scale = w.cash0, w.hmax, w.cost, w.sigma, w.reward_scale
    for i in range(4):
        c.obs_scale[i] = w.obs_scale[i]
    return c


def workspace_bytes(cfg: PrConfig) -> int:
    n = C.c_size_t()
    _check(lib().rollout_workspace_bytes(C.byref(cfg), C.byref(n)), "rollout_workspace_bytes")
    return n.value


def kernel_lds_bytes(cfg: PrConfig, with_actor: bool = True) -> int:
    """LDS bytes per workgroup of the persistent rollout kernel for this config (raises where it is not covered)."""
    n = C.c_size_t()
    _check(lib().rollout_kernel_lds_bytes(C.byref(cfg), int(with_actor), C.byref(n)), "rollout_kernel_lds_bytes")
    return n.value


def _weights_struct(net: Dict[str, torch.Tensor], P, S, Hd, O) -> PrWeights:
    shapes = {"W1": (P, S, Hd), "b1": (P, Hd), "W2": (P, Hd, Hd), "b2": (P, Hd), "W3": (P, Hd, O), "b3": (P, O)}
    w = PrWeights()
    for k, shp in shapes.items():
        setattr(w, k, _dev(net[k], torch.float32, shp, k))
    return w


class Rollout:
    """One rollout worker: owns the device workspace and keeps inputs alive."""

    def __init__(self, cfg: PrConfig, price: torch.Tensor, ind: Optional[torch.Tensor],
                 actor: Dict[str, torch.Tensor], critic: Dict[str, torch.Tensor]):
        self.cfg = cfg
        N, P, D, K, Hd = cfg.n_envs, cfg.n_agents, cfg.n_stocks, cfg.n_ind, cfg.hidden
        self.N, self.P, self.D, self.K, self.Hd = N, P, D, K, Hd
        self.S = 1 + 2 * D + D * K
        H, M = cfg.horizon, cfg.n_market
        nbytes = workspace_bytes(cfg)
        self._keep = (price, ind, actor, critic)
        m = PrMarket()
        m.price = _dev(price, torch.float32, (H + 1, M, D), "price")
        m.ind = _dev(ind, torch.float32, (H + 1, M, D * K), "ind") if K > 0 else None
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=price.device)
        ws = (self.workspace.data_ptr() + 255) // 256 * 256
        wa = _weights_struct(actor, P, self.S, Hd, D)
        wc = _weights_struct(critic, P, self.S, Hd, 1)
        self._h = C.c_void_p()
        _check(lib().rollout_init(C.byref(cfg), C.byref(m), C.byref(wa), C.byref(wc), ws, nbytes, _stream_ptr(),
                                  C.byref(self._h)), "rollout_init")
        self.device = price.device

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().rollout_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_weights(self, actor, critic):
        wa = _weights_struct(actor, self.P, self.S, self.Hd, self.D)
        wc = _weights_struct(critic, self.P, self.S, self.Hd, 1)
        _check(lib().rollout_set_weights(self._h, C.byref(wa), C.byref(wc)), "rollout_set_weights")
        self._keep = self._keep[:2] + (actor, critic)

    def reset(self):
        _check(lib().rollout_reset(self._h), "rollout_reset")

    def set_replay(self, price: torch.Tensor, ind: Optional[torch.Tensor], start: torch.Tensor):
        """Episodes of env n run over rows start[n] .. start[n] + H of the table price [rows, M, D], ind [rows, M, D*K]."""
        rows = int(price.shape[0])
        m = PrMarket()
        m.price = _dev(price, torch.float32, (rows, self.cfg.n_market, self.D), "price")
        m.ind = _dev(ind, torch.float32, (rows, self.cfg.n_market, self.D * self.K), "ind") if self.K > 0 else None
        s = _dev(start, torch.int32, (self.N,), "start")
        _check(lib().rollout_set_replay(self._h, C.byref(m), rows, s), "rollout_set_replay")
        self._keep = (price, ind) + self._keep[2:]

    def alloc_buffers(self, T: int, value=True, logp=True, mu=False, shares=False) -> Dict[str, torch.Tensor]:
        N, D, S, dev = self.N, self.D, self.S, self.device
        e = lambda shp, dt: torch.empty(shp, dtype=dt, device=dev)
        out = {"obs": e((T + 1, N, S), torch.float32), "act_raw": e((T, N, D), torch.float32),
               "reward": e((T, N), torch.float32), "done": e((T, N), torch.uint8)}
        if value:
            out["value"] = e((T + 1, N), torch.float32)
        if logp:
            out["logp"] = e((T, N), torch.float32)
        if mu:
            out["mu"] = e((T, N, D), torch.float32)
        if shares:
            out["shares"] = e((T, N, D), torch.int32)
        return out

    def _buffers(self, T: int, out: Dict[str, torch.Tensor]) -> PrBuffers:
        N, D, S = self.N, self.D, self.S
        spec = {"obs": (torch.float32, (T + 1, N, S)), "act_raw": (torch.float32, (T, N, D)),
                "reward": (torch.float32, (T, N)), "done": (torch.uint8, (T, N)),
                "value": (torch.float32, (T + 1, N)), "logp": (torch.float32, (T, N)),
                "mu": (torch.float32, (T, N, D)), "shares": (torch.int32, (T, N, D))}
        b = PrBuffers()
        for k, (dt, shp) in spec.items():
            setattr(b, k, _dev(out[k], dt, shp, k) if out.get(k) is not None else None)
        return b

    def step_T(self, T: int, noise: torch.Tensor, out: Dict[str, torch.Tensor]):
        b = self._buffers(T, out)
        _check(lib().rollout_step_T(self._h, T, _dev(noise, torch.float32, (T, self.N, self.D), "noise"),
                                    C.byref(b)), "rollout_step_T")
        return out

    def step_forced(self, T: int, mu: torch.Tensor, noise: torch.Tensor, out: Dict[str, torch.Tensor]):
        b = self._buffers(T, out)
        shp = (T, self.N, self.D)
        _check(lib().rollout_step_forced(self._h, T, _dev(mu, torch.float32, shp, "mu"),
                                         _dev(noise, torch.float32, shp, "noise"), C.byref(b)),
               "rollout_step_forced")
        return out

    def mlp_forward(self, net: int, X: torch.Tensor, Y: Optional[torch.Tensor] = None) -> torch.Tensor:
        if X.dim() != 2 or X.stride(1) != 1 or X.dtype != torch.float32 or not X.is_cuda:
            raise TypeError("X: need a 2-d float32 cuda tensor with unit column stride")
        rows, ldx = X.shape[0], X.stride(0)
        O = self.D if net == PR_NET_ACTOR else 1
        if Y is None:
            Y = torch.empty((rows, O), dtype=torch.float32, device=X.device)
        _dev(Y, torch.float32, (rows, O), "Y")
        _check(lib().rollout_mlp_forward(self._h, net, rows, X.data_ptr(), ldx, Y.data_ptr()), "rollout_mlp_forward")
        return Y

    def _state_struct(self, st: Dict[str, torch.Tensor]) -> PrState:
        N, D = self.N, self.D
        spec = {"cash": (torch.float32, (N,)), "holdings": (torch.int32, (N, D)), "cursor": (torch.int32, (N,)),
                "ep_return": (torch.float64, (N,)), "ep_sum": (torch.float64, (N,)),
                "ep_sqsum": (torch.float64, (N,)), "ep_count": (torch.int32, (N,))}
        s = PrState()
        for k, (dt, shp) in spec.items():
            setattr(s, k, _dev(st[k], dt, shp, k) if st.get(k) is not None else None)
        return s

    def get_state(self) -> Dict[str, torch.Tensor]:
        N, D, dev = self.N, self.D, self.device
        st = {"cash": torch.empty(N, dtype=torch.float32, device=dev),
              "holdings": torch.empty((N, D), dtype=torch.int32, device=dev),
              "cursor": torch.empty(N, dtype=torch.int32, device=dev),
              "ep_return": torch.empty(N, dtype=torch.float64, device=dev),
              "ep_sum": torch.empty(N, dtype=torch.float64, device=dev),
              "ep_sqsum": torch.empty(N, dtype=torch.float64, device=dev),
              "ep_count": torch.empty(N, dtype=torch.int32, device=dev)}
        s = self._state_struct(st)
        _check(lib().rollout_get_state(self._h, C.byref(s)), "rollout_get_state")
        return st

    def set_state(self, st: Dict[str, torch.Tensor]):
        s = self._state_struct(st)
        _check(lib().rollout_set_state(self._h, C.byref(s)), "rollout_set_state")

    def leaderboard(self):
        dev = self.device
        mean = torch.empty(self.P, dtype=torch.float64, device=dev)
        var = torch.empty(self.P, dtype=torch.float64, device=dev)
        rank = torch.empty(self.P, dtype=torch.int32, device=dev)
        _check(lib().rollout_leaderboard(self._h, mean.data_ptr(), var.data_ptr(), rank.data_ptr()),
               "rollout_leaderboard")
        return mean, var, rank


def compute_gae(reward: torch.Tensor, value: torch.Tensor, done: torch.Tensor, gamma: float, lam: float,
                adv: Optional[torch.Tensor] = None, ret: Optional[torch.Tensor] = None):
    T, N = reward.shape
    if adv is None:
        adv = torch.empty_like(reward)
    if ret is None:
        ret = torch.empty_like(reward)
    _check(lib().compute_gae(_stream_ptr(), T, N, _dev(reward, torch.float32, (T, N), "reward"),
                             _dev(value, torch.float32, (T + 1, N), "value"), _dev(done, torch.uint8, (T, N), "done"),
                             gamma, lam, _dev(adv, torch.float32, (T, N), "adv"),
                             _dev(ret, torch.float32, (T, N), "ret")), "compute_gae")
    return adv, ret


METRICS = ("cumulative_return", "annual_return", "annual_volatility", "max_drawdown", "sharpe", "calmar")


def trading_metrics(obs: torch.Tensor, done: torch.Tensor, n_stocks: int, obs_scale, periods_per_year: float,
                    risk_free: float = 0.0):
    """obs [T+1, N, S], done [T, N] of a recorded rollout -> (metrics [6, N] float64 in the order of METRICS,
    length [N] int32) for the first episode of every env."""
    T1, N, S = obs.shape
    T = T1 - 1
    out = torch.empty((6, N), dtype=torch.float64, device=obs.device)
    length = torch.empty((N,), dtype=torch.int32, device=obs.device)
    sc = (C.c_float * 4)(*[float(x) for x in obs_scale])
    _check(lib().trading_metrics(_stream_ptr(), T, N, int(n_stocks), S, _dev(obs, torch.float32, (T1, N, S), "obs"),
                                 _dev(done, torch.uint8, (T, N), "done"), sc, float(periods_per_year),
                                 float(risk_free), _dev(out, torch.float64, (6, N), "metrics"),
                                 _dev(length, torch.int32, (N,), "length")), "trading_metrics")
    return out, length


def population_refill(params: torch.Tensor, rank: torch.Tensor, keep: int, sigma: float = 0.0,
                      noise: Optional[torch.Tensor] = None) -> torch.Tensor:
    """In place on params [P, ...]: agents ranked behind the first `keep` become copies of the kept ones (in turn)
    plus sigma * noise.  rank: int32 [P], best first."""
    P = params.shape[0]
    count = params.numel() // P
    shape = tuple(params.shape)
    _check(lib().population_refill(_stream_ptr(), P, count, _dev(rank, torch.int32, (P,), "rank"), int(keep),
                                   float(sigma), None if noise is None else _dev(noise, torch.float32, shape, "noise"),
                                   _dev(params, torch.float32, shape, "params")), "population_refill")
    return params


# ------------------------------------------------------------------ learner

NET_KEYS = ("W1", "b1", "W2", "b2", "W3", "b3")


def make_ppo_config(w, batch: int = 1024, clip: float = 0.2, value_coef: float = 0.5, lr: float = 1e-3,
                    beta1: float = 0.9, beta2: float = 0.999, adam_eps: float = 1e-8, adam_step: int = 1) -> PrPpoConfig:
    """Batch size and learning rate default to the paper's (Sec. 5.2)."""
    return PrPpoConfig(batch, w.n_stocks, w.n_ind, w.hidden, w.sigma, clip, value_coef, lr, beta1, beta2, adam_eps,
                       adam_step)


def _net_shapes(cfg: PrPpoConfig, out_dim: int):
    S, Hd = 1 + 2 * cfg.n_stocks + cfg.n_stocks * cfg.n_ind, cfg.hidden
    return {"W1": (S, Hd), "b1": (Hd,), "W2": (Hd, Hd), "b2": (Hd,), "W3": (Hd, out_dim), "b3": (out_dim,)}


def _net_struct(net: Dict[str, torch.Tensor], cfg: PrPpoConfig, out_dim: int, what: str) -> PrNetParams:
    shp = _net_shapes(cfg, out_dim)
    return PrNetParams(*[_dev(net[k], torch.float32, shp[k], f"{what}.{k}") for k in NET_KEYS])


def ppo_workspace(cfg: PrPpoConfig, device) -> torch.Tensor:
    n = C.c_size_t(0)
    _check(lib().ppo_workspace_bytes(C.byref(cfg), C.byref(n)), "ppo_workspace_bytes")
    return torch.empty(n.value + 256, dtype=torch.uint8, device=device)


def _aligned_ptr(ws: torch.Tensor):
    p = (ws.data_ptr() + 255) // 256 * 256
    return p, ws.numel() - (p - ws.data_ptr())


def _batch_args(cfg, obs, act_raw, logp_old, adv, ret, rows):
    R = obs.shape[0]
    S, D = 1 + 2 * cfg.n_stocks + cfg.n_stocks * cfg.n_ind, cfg.n_stocks
    return [_dev(obs, torch.float32, (R, S), "obs"), _dev(act_raw, torch.float32, (R, D), "act_raw"),
            _dev(logp_old, torch.float32, (R,), "logp_old"), _dev(adv, torch.float32, (R,), "adv"),
            _dev(ret, torch.float32, (R,), "ret"),
            None if rows is None else _dev(rows, torch.int32, (cfg.batch,), "rows")]


def ppo_minibatch_grads(cfg: PrPpoConfig, obs, act_raw, logp_old, adv, ret, rows, actor, critic, workspace=None):
    """Gradients of the PPO objective for one minibatch: (grads_actor, grads_critic, stats[4]) as device tensors."""
    dev = obs.device
    ws = ppo_workspace(cfg, dev) if workspace is None else workspace
    ptr, nbytes = _aligned_ptr(ws)
    ga = {k: torch.empty(v, dtype=torch.float32, device=dev) for k, v in _net_shapes(cfg, cfg.n_stocks).items()}
    gc = {k: torch.empty(v, dtype=torch.float32, device=dev) for k, v in _net_shapes(cfg, 1).items()}
    stats = torch.empty(4, dtype=torch.float32, device=dev)
    sa, sc = _net_struct(actor, cfg, cfg.n_stocks, "actor"), _net_struct(critic, cfg, 1, "critic")
    sga, sgc = _net_struct(ga, cfg, cfg.n_stocks, "grad_actor"), _net_struct(gc, cfg, 1, "grad_critic")
    _check(lib().ppo_minibatch_grads(_stream_ptr(), C.byref(cfg), *_batch_args(cfg, obs, act_raw, logp_old, adv, ret, rows),
                                     C.byref(sa), C.byref(sc), C.byref(sga), C.byref(sgc), ptr, nbytes,
                                     stats.data_ptr()), "ppo_minibatch_grads")
    return ga, gc, stats


def ppo_minibatch_grads_noalloc(cfg: PrPpoConfig, obs, act_raw, logp_old, adv, ret, rows, actor, critic, grad_actor,
                                grad_critic, stats):
    """The same gradients through the entry point that owns its scratch: every output tensor is the caller's."""
    sa, sc = _net_struct(actor, cfg, cfg.n_stocks, "actor"), _net_struct(critic, cfg, 1, "critic")
    sga, sgc = _net_struct(grad_actor, cfg, cfg.n_stocks, "grad_actor"), _net_struct(grad_critic, cfg, 1, "grad_critic")
    _check(lib().ppo_minibatch_grads_noalloc(_stream_ptr(), C.byref(cfg),
                                             *_batch_args(cfg, obs, act_raw, logp_old, adv, ret, rows), C.byref(sa),
                                             C.byref(sc), C.byref(sga), C.byref(sgc),
                                             _dev(stats, torch.float32, (4,), "stats")), "ppo_minibatch_grads_noalloc")
    return grad_actor, grad_critic, stats


def adam_update(theta, grad, m, v, lr, beta1, beta2, eps, t):
    n = theta.numel()
    shp = tuple(theta.shape)
    _check(lib().adam_update(_stream_ptr(), n, _dev(theta, torch.float32, shp, "theta"),
                             _dev(grad, torch.float32, shp, "grad"), _dev(m, torch.float32, shp, "m"),
                             _dev(v, torch.float32, shp, "v"), lr, beta1, beta2, eps, int(t)), "adam_update")
    return theta


def ppo_learner_step(cfg: PrPpoConfig, obs, act_raw, logp_old, adv, ret, rows, actor, critic, m_actor, v_actor,
                     m_critic, v_critic, workspace):
    """One optimiser step in place on actor / critic and their Adam moments; returns stats[4] (device)."""
    ptr, nbytes = _aligned_ptr(workspace)
    stats = torch.empty(4, dtype=torch.float32, device=obs.device)
    D = cfg.n_stocks
    st = [_net_struct(actor, cfg, D, "actor"), _net_struct(critic, cfg, 1, "critic"),
          _net_struct(m_actor, cfg, D, "m_actor"), _net_struct(v_actor, cfg, D, "v_actor"),
          _net_struct(m_critic, cfg, 1, "m_critic"), _net_struct(v_critic, cfg, 1, "v_critic")]
    _check(lib().ppo_learner_step(_stream_ptr(), C.byref(cfg), *_batch_args(cfg, obs, act_raw, logp_old, adv, ret, rows),
                                  *[C.byref(x) for x in st], ptr, nbytes, stats.data_ptr()), "ppo_learner_step")
    return stats


# -------------------------------------------------------------- calibration

PR_CAL_COPY, PR_CAL_READ, PR_CAL_PROBE = 0, 1, 2
ROLE_NONE, ROLE_MATRIX, ROLE_VECTOR, ROLE_BOTH, ROLE_PLAIN = 0, 1, 2, 3, 4


def calibrate_stream(kind: int, src: torch.Tensor, dst: torch.Tensor):
    """One streaming launch over all of src (copy into dst, or read only); the caller times it."""
    n = src.numel() * src.element_size()
    _check(lib().rollout_calibrate(_stream_ptr(), kind, n, None, src.data_ptr(), dst.data_ptr()), "rollout_calibrate")


def calibrate_probe(roles, iters_matrix: int, iters_vector: int, acts_per_group: int = 0, lds_reads: bool = False,
                    blocks: int = 256, ticks: Optional[torch.Tensor] = None):
    """One launch of the matrix / vector co-issue probe: roles = 8 ROLE_* values, one per wavefront of a workgroup.
    Returns ticks [blocks, 8] (int64, 10 ns units; -1 where a wavefront had no role)."""
    assert len(roles) == 8
    if ticks is None:
        ticks = torch.full((blocks, 8), -1, dtype=torch.int64, device="cuda")
    sink = torch.zeros(4, dtype=torch.float32, device=ticks.device)
    params = (C.c_int32 * 12)(*roles, iters_matrix, iters_vector, acts_per_group, int(lds_reads))
    _check(lib().rollout_calibrate(_stream_ptr(), PR_CAL_PROBE, blocks, params, ticks.data_ptr(), sink.data_ptr()),
           "rollout_calibrate")
    return ticks
