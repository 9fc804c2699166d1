"""ctypes front end of the CPU checker in podoracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the bench's
CPU-baseline leg.  The product package never imports this module, and this
module never imports the product package.

All functions take and return numpy arrays in the logical layouts of the C
file ([T, N, D] etc.).  Real-valued results come back in float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "podoracle.c")
_LIB = os.path.join(_HERE, "libpodoracle.so")

FLAG_TRUNC, FLAG_FLOOR, FLAG_GUARD = 1, 2, 4


def build(force: bool = False) -> str:
    """Compile podoracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Cfg(C.Structure):
    _fields_ = [("n_stocks", C.c_int32), ("n_ind", C.c_int32), ("horizon", C.c_int32),
                ("cash0", C.c_float), ("hmax", C.c_float), ("cost", C.c_float), ("sigma", C.c_float),
                ("reward_scale", C.c_float), ("obs_scale", C.c_float * 4)]


class _State(C.Structure):
    _fields_ = [("cash", C.c_void_p), ("h", C.c_void_p), ("tau", C.c_void_p), ("asset", C.c_void_p),
                ("ep_ret", C.c_void_p), ("ep_sum", C.c_void_p), ("ep_sqsum", C.c_void_p), ("ep_cnt", C.c_void_p),
                ("start", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_bf16_round.restype = C.c_float
        _lib.orc_bf16_round.argtypes = [C.c_float]
        _lib.orc_asset.restype = C.c_double
        _lib.orc_env_step.restype = C.c_double
        _lib.orc_rollout.restype = C.c_int
    return _lib


def make_cfg(n_stocks, n_ind, horizon, cash0=1e6, hmax=100.0, cost=1e-3, sigma=0.5,
             reward_scale=2.0 ** -12, obs_scale=(2.0 ** -20, 2.0 ** -7, 2.0 ** -10, 1.0)) -> Cfg:
    c = Cfg()
    c.n_stocks, c.n_ind, c.horizon = int(n_stocks), int(n_ind), int(horizon)
    c.cash0, c.hmax, c.cost, c.sigma, c.reward_scale = cash0, hmax, cost, sigma, reward_scale
    for i in range(4):
        c.obs_scale[i] = obs_scale[i]
    return c


def cfg_from_workload(w, horizon: Optional[int] = None) -> Cfg:
    """Build the constants from any object with the workload's field names."""
    return make_cfg(w.n_stocks, w.n_ind, w.steps if horizon is None else horizon, w.cash0, w.hmax, w.cost,
                    w.sigma, w.reward_scale, w.obs_scale)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def bf16_round(x) -> np.ndarray:
    x = _f32(x)
    out = np.empty_like(x)
    lib().orc_bf16_round_array(_p(x), _p(out), C.c_int64(x.size))
    return out


def mlp(X, W1, b1, W2, b2, W3, b3, out_tanh: bool, bf16: bool) -> np.ndarray:
    """Rows of X [rows, S] through one agent's network; float64 [rows, O].

    With bf16=True the weights are rounded here, once, before use."""
    X = _f32(X)
    rows, S = X.shape
    ws = [_f32(a) for a in (W1, b1, W2, b2, W3, b3)]
    Hd = ws[0].shape[1]
    O = ws[4].shape[1]
    assert ws[0].shape == (S, Hd) and ws[2].shape == (Hd, Hd) and ws[4].shape == (Hd, O)
    if bf16:
        ws[0], ws[2], ws[4] = bf16_round(ws[0]), bf16_round(ws[2]), bf16_round(ws[4])
    out = np.empty((rows, O), dtype=np.float64)
    lib().orc_mlp(C.c_int64(rows), S, Hd, O, _p(X), C.c_int64(S), *[_p(a) for a in ws], int(out_tanh), int(bf16),
                  _p(out))
    return out


def observe(cfg: Cfg, cash: float, h, p, ind) -> np.ndarray:
    D, K = cfg.n_stocks, cfg.n_ind
    h = np.ascontiguousarray(h, dtype=np.int32)
    p, ind = _f32(p), _f32(ind)
    obs = np.empty(1 + 2 * D + D * K, dtype=np.float32)
    lib().orc_observe(C.byref(cfg), C.c_float(cash), _p(h), _p(p), _p(ind), _p(obs))
    return obs


def sample(sigma: float, mu, eps):
    mu, eps = _f32(mu), _f32(eps)
    a = np.empty_like(mu)
    lp = C.c_double()
    lib().orc_sample(int(mu.size), C.c_float(sigma), _p(mu), _p(eps), _p(a), C.byref(lp))
    return a, lp.value


def trade(cfg: Cfg, cash: float, h, a_raw, p):
    """One env's trade execution.  Returns (cash', h', shares, flags)."""
    h = np.array(h, dtype=np.int32)
    a_raw, p = _f32(a_raw), _f32(p)
    shares = np.empty(cfg.n_stocks, dtype=np.int32)
    flags = np.empty(cfg.n_stocks, dtype=np.uint8)
    c = C.c_float(cash)
    lib().orc_trade(C.byref(cfg), C.byref(c), _p(h), _p(a_raw), _p(p), _p(shares), _p(flags))
    return np.float32(c.value), h, shares, flags


def asset(cash: float, h, p) -> float:
    h = np.ascontiguousarray(h, dtype=np.int32)
    p = _f32(p)
    return lib().orc_asset(int(h.size), C.c_float(cash), _p(h), _p(p))


class State:
    """Persistent per-env state (cash, holdings, cursor, asset, episode sums)."""

    def __init__(self, cfg: Cfg, n_envs: int, start=None):
        """start: per-env table row where every episode of the env begins (None = row 0)."""
        D = cfg.n_stocks
        self.n_envs = n_envs
        self.start = np.zeros(n_envs, dtype=np.int32) if start is None else np.array(start, dtype=np.int32)
        assert self.start.shape == (n_envs,) and (self.start >= 0).all()
        self.cash = np.empty(n_envs, dtype=np.float32)
        self.h = np.empty((n_envs, D), dtype=np.int32)
        self.tau = np.empty(n_envs, dtype=np.int32)
        self.asset = np.empty(n_envs, dtype=np.float64)
        self.ep_ret = np.empty(n_envs, dtype=np.float64)
        self.ep_sum = np.empty(n_envs, dtype=np.float64)
        self.ep_sqsum = np.empty(n_envs, dtype=np.float64)
        self.ep_cnt = np.empty(n_envs, dtype=np.int32)
        lib().orc_reset_state(C.byref(cfg), C.c_int64(n_envs), C.byref(self._c()))

    def _c(self) -> _State:
        s = _State()
        for name, _ in _State._fields_:
            setattr(s, name, getattr(self, name).ctypes.data)
        return s


def env_step(cfg: Cfg, state: State, n: int, a_raw, p_now, p_next):
    """One transition of env n of `state`.  Returns (reward, done, shares, flags)."""
    a_raw, p_now, p_next = _f32(a_raw), _f32(p_now), _f32(p_next)
    shares = np.empty(cfg.n_stocks, dtype=np.int32)
    flags = np.empty(cfg.n_stocks, dtype=np.uint8)
    done = C.c_uint8()
    cs = state._c()
    r = lib().orc_env_step(C.byref(cfg), C.c_int64(n), C.byref(cs), _p(a_raw), _p(p_now), _p(p_next), _p(shares),
                           _p(flags), C.byref(done))
    return r, int(done.value), shares, flags


def _net_ptrs(net: Optional[Dict[str, np.ndarray]], bf16: bool):
    if net is None:
        return None, None
    arrs = [_f32(net[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]
    if bf16:
        for i in (0, 2, 4):
            arrs[i] = bf16_round(arrs[i])
    ptrs = (C.c_void_p * 6)(*[a.ctypes.data for a in arrs])
    return ptrs, arrs


def rollout(cfg: Cfg, hidden: int, bf16: bool, T: int, price, ind, noise, actor=None, critic=None,
            mu_forced=None, state: Optional[State] = None, agent_of=None, market_of=None,
            want=("obs", "mu", "act_raw", "logp", "reward", "done", "value", "shares", "flags")):
    """Free-running (actor given) or teacher-forced (mu_forced given) rollout.

    price [H+1, M, D], ind [H+1, M, D*K], noise [T, N, D]; nets are dicts with
    a leading agent axis.  Returns (dict of outputs, state)."""
    price, ind, noise = _f32(price), _f32(ind), _f32(noise)
    N, D = noise.shape[1], cfg.n_stocks
    M = price.shape[1]
    S = 1 + 2 * D + D * cfg.n_ind
    assert noise.shape == (T, N, D) and ind.shape[:2] == price.shape[:2]
    if state is None:
        state = State(cfg, N)
    assert price.shape[0] >= int(state.start.max()) + cfg.horizon + 1
    agent_of = np.zeros(N, dtype=np.int32) if agent_of is None else np.ascontiguousarray(agent_of, dtype=np.int32)
    if market_of is None:
        market_of = np.arange(N, dtype=np.int32) % M
    market_of = np.ascontiguousarray(market_of, dtype=np.int32)
    a_ptr, a_keep = _net_ptrs(actor, bf16)
    c_ptr, c_keep = _net_ptrs(critic, bf16)
    if mu_forced is not None:
        mu_forced = _f32(mu_forced)
        assert mu_forced.shape == (T, N, D)
    else:
        assert actor is not None
    out = {}
    shp = {"obs": ((T + 1, N, S), np.float32), "mu": ((T, N, D), np.float64), "act_raw": ((T, N, D), np.float32),
           "logp": ((T, N), np.float64), "reward": ((T, N), np.float64), "done": ((T, N), np.uint8),
           "value": ((T + 1, N), np.float64), "shares": ((T, N, D), np.int32), "flags": ((T, N, D), np.uint8)}
    for k in want:
        if k == "value" and critic is None:
            continue
        out[k] = np.empty(*shp[k])
    g = lambda k: _p(out.get(k))
    cs = state._c()
    rc = lib().orc_rollout(C.byref(cfg), C.c_int64(N), int(M), int(hidden), int(bf16), int(T), _p(agent_of),
                           _p(market_of), _p(price), _p(ind), a_ptr, c_ptr, _p(noise), _p(mu_forced), C.byref(cs),
                           g("obs"), g("mu"), g("act_raw"), g("logp"), g("reward"), g("done"), g("value"),
                           g("shares"), g("flags"))
    if rc != 0:
        raise MemoryError("orc_rollout")
    del a_keep, c_keep
    return out, state


def gae(reward, value, done, gamma: float, lam: float):
    reward = np.ascontiguousarray(reward, dtype=np.float64)
    value = np.ascontiguousarray(value, dtype=np.float64)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    T, N = reward.shape
    assert value.shape == (T + 1, N) and done.shape == (T, N)
    adv = np.empty((T, N), dtype=np.float64)
    ret = np.empty((T, N), dtype=np.float64)
    lib().orc_gae(int(T), C.c_int64(N), _p(reward), _p(value), _p(done), C.c_double(gamma), C.c_double(lam), _p(adv),
                  _p(ret))
    return adv, ret


def leaderboard(n_agents: int, agent_of, ep_sum, ep_sqsum, ep_cnt):
    agent_of = np.ascontiguousarray(agent_of, dtype=np.int32)
    ep_sum = np.ascontiguousarray(ep_sum, dtype=np.float64)
    ep_sqsum = np.ascontiguousarray(ep_sqsum, dtype=np.float64)
    ep_cnt = np.ascontiguousarray(ep_cnt, dtype=np.int32)
    mean = np.empty(n_agents, dtype=np.float64)
    var = np.empty(n_agents, dtype=np.float64)
    rank = np.empty(n_agents, dtype=np.int32)
    lib().orc_leaderboard(int(n_agents), C.c_int64(agent_of.size), _p(agent_of), _p(ep_sum), _p(ep_sqsum), _p(ep_cnt),
                          _p(mean), _p(var), _p(rank))
    return mean, var, rank


def asset_curve(obs, done, n_stocks: int, obs_scale):
    """Value curve of the first episode of every env, decoded from a recorded observation buffer."""
    obs = np.ascontiguousarray(obs, dtype=np.float32)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    T1, N, S = obs.shape
    T = T1 - 1
    assert done.shape == (T, N)
    sc = np.ascontiguousarray(obs_scale, dtype=np.float32)
    value = np.empty((T + 1, N), dtype=np.float64)
    length = np.empty(N, dtype=np.int32)
    lib().orc_asset_curve(int(T), C.c_int64(N), int(n_stocks), int(S), _p(obs), _p(done), _p(sc), _p(value), _p(length))
    return value, length


def metrics(value, length, periods_per_year: float, rf: float = 0.0):
    """[6, N]: cumulative return, annual return, annual volatility, max drawdown, Sharpe, Calmar (Sec. 5.3)."""
    value = np.ascontiguousarray(value, dtype=np.float64)
    length = np.ascontiguousarray(length, dtype=np.int32)
    T1, N = value.shape
    out = np.empty((6, N), dtype=np.float64)
    lib().orc_metrics(int(T1 - 1), C.c_int64(N), _p(value), _p(length), C.c_double(periods_per_year), C.c_double(rf),
                      _p(out))
    return out


def population_refill(params, rank, keep: int, sigma: float, noise=None):
    """Returns the refilled copy of params [P, count] (Sec. 4.1 generator: losers <- candidates + mutation)."""
    out = np.array(params, dtype=np.float32, order="C", copy=True)
    P = out.shape[0]
    flat = out.reshape(P, -1)
    rank = np.ascontiguousarray(rank, dtype=np.int32)
    z = None if noise is None else np.ascontiguousarray(noise, dtype=np.float32).reshape(P, -1)
    assert rank.shape == (P,) and 1 <= keep <= P and (z is None or z.shape == flat.shape)
    lib().orc_population_refill(int(P), C.c_int64(flat.shape[1]), _p(rank), int(keep), C.c_float(sigma), _p(z), _p(flat))
    return out


NET_KEYS = ("W1", "b1", "W2", "b2", "W3", "b3")


def ppo_grads(obs, act, logp_old, adv, ret, actor, critic, sigma: float, clip: float, value_coef: float):
    """One PPO minibatch in fp64: returns (grads_actor, grads_critic, stats[4], margin[B]); nets are dicts of fp32
    arrays without an agent axis (W [in, out])."""
    obs, act = _f32(obs), _f32(act)
    B, S = obs.shape
    D = act.shape[1]
    Hd = actor["W1"].shape[1]
    a = {k: _f32(actor[k]) for k in NET_KEYS}
    c = {k: _f32(critic[k]) for k in NET_KEYS}
    assert a["W1"].shape == (S, Hd) and a["W3"].shape == (Hd, D) and c["W3"].shape == (Hd, 1)
    ga = {k: np.zeros(a[k].shape, np.float64) for k in NET_KEYS}
    gc = {k: np.zeros(c[k].shape, np.float64) for k in NET_KEYS}
    stats = np.zeros(4, np.float64)
    margin = np.zeros(B, np.float64)
    lib().orc_ppo_grads(int(B), int(S), int(Hd), int(D), _p(obs), _p(act), _p(_f32(logp_old)), _p(_f32(adv)),
                        _p(_f32(ret)), *[_p(a[k]) for k in NET_KEYS], *[_p(c[k]) for k in NET_KEYS],
                        C.c_double(sigma), C.c_double(clip), C.c_double(value_coef),
                        *[_p(ga[k]) for k in NET_KEYS], *[_p(gc[k]) for k in NET_KEYS], _p(stats), _p(margin))
    return ga, gc, stats, margin


def adam(theta, g, m, v, lr: float, b1: float, b2: float, eps: float, t: int):
    """In fp64; returns new (theta, m, v)."""
    theta, m, v = (np.array(x, dtype=np.float64, copy=True) for x in (theta, m, v))
    g = np.ascontiguousarray(g, dtype=np.float64)
    lib().orc_adam(C.c_int64(theta.size), _p(theta), _p(g), _p(m), _p(v), C.c_double(lr), C.c_double(b1),
                   C.c_double(b2), C.c_double(eps), int(t))
    return theta, m, v
