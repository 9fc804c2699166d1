"""Stage-wise comparison of a GPU rollout record with the CPU checker.

The map from the policy mean to the trajectory is discontinuous (share counts
are truncated), so stages are compared with their inputs taken from the GPU's
own record: the networks on the recorded observations, the environment on the
recorded means and noise.

Tolerances.  Integers and everything that is an exact function of them are
compared bit for bit.  Network outputs are held to two tiers:

  normwise    max |got - want| <= TOL_NORM * (largest |entry| of the output
              vector the value belongs to): the row for the actor, the
              compared batch for the scalar critic.  1e-5 for fp32 operands,
              1e-2 for bf16 operands.
  entry-wise  |got - want| <= TOL_ENTRY * |want| on every entry that is not
              small next to that largest entry: 1e-4 (the stated fp32
              tolerance) on entries >= 0.1 of it, 2e-2 (the stated bf16
              tolerance) on entries >= 0.5 of it.

A purely entry-wise relative error is not meaningful near zero: binary32
accumulation over 301 + 256 + 256 terms leaves an absolute error of a few 1e-6
on outputs of size 1 whatever the entry, and with bf16 activations a one-ulp
re-quantisation flip in the first hidden layer moves every output by a few
1e-3.  Every check records the worst ratios it saw in WORST (printed by the
tests), so the slack of the bounds can be read from a test run.
"""
from __future__ import annotations

import numpy as np

import oracle

TOL_F32 = 1e-4            # stated tolerance of the fp32 path (entry-wise tier; also used for log-probs, GAE, gradients)
TOL_BF16 = 2e-2           # stated tolerance of the bf16 path (entry-wise tier)
TOL_NORM_F32 = 1e-5       # normwise tier
TOL_NORM_BF16 = 1e-2
ENTRY_FLOOR_F32 = 0.1     # entry-wise tier applies to entries >= floor * largest entry
ENTRY_FLOOR_BF16 = 0.5

WORST = {}                # name -> largest (observed error / allowed error) over the process


def to_np(t):
    return t.detach().cpu().numpy()


def rel_err_rows(got, want):
    """max |got - want| / (largest |want| of the same row), rows = last axis."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    scale = np.maximum(np.abs(want).max(axis=-1, keepdims=True), 1e-30)
    return float((np.abs(got - want) / scale).max())


def _note(name, ratio):
    WORST[name] = max(WORST.get(name, 0.0), float(ratio))


def check_two_tier(name, got, want, bf16):
    """got, want [R, C]: both tiers, rows = output vectors.  Returns (normwise error, entry-wise error)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape and got.ndim == 2
    tol_n, tol_e, floor = ((TOL_NORM_BF16, TOL_BF16, ENTRY_FLOOR_BF16) if bf16 else
                           (TOL_NORM_F32, TOL_F32, ENTRY_FLOOR_F32))
    err = np.abs(got - want)
    top = np.maximum(np.abs(want).max(axis=1, keepdims=True), 1e-30)
    e_norm = float((err / top).max())
    big = np.abs(want) >= floor * top
    e_entry = float((err[big] / np.abs(want)[big]).max()) if big.any() else 0.0
    _note(name + ".normwise", e_norm / tol_n)
    _note(name + ".entrywise", e_entry / tol_e)
    assert e_norm <= tol_n, f"{name}: normwise error {e_norm:.3e} > {tol_n:.0e}"
    assert e_entry <= tol_e, f"{name}: entry-wise error {e_entry:.3e} > {tol_e:.0e} on entries >= {floor} of the largest"
    return e_norm, e_entry


def check_networks(w, weights_actor, weights_critic, obs_rows, mu_rows=None, value_rows=None, agent=0):
    """obs_rows [R, S] from the GPU record -> checker outputs vs recorded mu / value of the same rows."""
    bf16 = bool(w.mlp_dtype)
    errs = {}
    if mu_rows is not None:
        a = {k: v[agent] for k, v in weights_actor.items()}
        want = oracle.mlp(obs_rows, a["W1"], a["b1"], a["W2"], a["b2"], a["W3"], a["b3"], True, bf16)
        errs["mu"] = check_two_tier("mu", np.asarray(mu_rows).reshape(want.shape), want, bf16)
    if value_rows is not None:
        c = {k: v[agent] for k, v in weights_critic.items()}
        want = oracle.mlp(obs_rows, c["W1"], c["b1"], c["W2"], c["b2"], c["W3"], c["b3"], False, bf16)
        # the critic has one output per row: the compared batch is the output vector, every value is an entry
        errs["value"] = check_two_tier("value", np.asarray(value_rows).reshape(1, -1), want.reshape(1, -1), bf16)
    return errs


def reward_tolerance(w, reward64):
    """|r_gpu - r_checker| <= 1e-4 |r| + 16 ulp32(cash0) rho: the absolute term is the
    binary32 representation error of a balance of the size of the initial capital."""
    return 1e-4 * np.abs(reward64) + 16.0 * float(np.spacing(np.float32(w.cash0))) * w.reward_scale


def check_env_record(w, cfg, rec, price, ind, noise, mu, state0=None, agent_of=None, market_of=None):
    """Teacher-forced on the recorded means: the checker replays the whole
    rollout from `state0` and must reproduce the GPU record.

    rec: dict of numpy arrays (obs, act_raw, reward, done, shares, logp).  Returns the checker's outputs."""
    T = rec["reward"].shape[0]
    out, st = oracle.rollout(cfg, w.hidden, bool(w.mlp_dtype), T, price, ind, noise, mu_forced=mu, state=state0,
                             agent_of=agent_of, market_of=market_of,
                             want=("obs", "act_raw", "logp", "reward", "done", "shares", "flags"))
    assert np.array_equal(rec["act_raw"].view(np.uint32), out["act_raw"].view(np.uint32)), "act_raw bits"
    assert np.array_equal(rec["done"], out["done"]), "done"
    if "shares" in rec:
        bad = rec["shares"] != out["shares"]
        if bad.any():
            flagged = out["flags"][bad] != 0
            raise AssertionError(f"{int(bad.sum())} share counts differ ({int(flagged.sum())} at flagged sites); "
                                 f"first at {np.argwhere(bad)[0].tolist()}")
    assert np.array_equal(rec["obs"].view(np.uint32), out["obs"].view(np.uint32)), "obs bits"
    tol = reward_tolerance(w, out["reward"])
    err = np.abs(rec["reward"].astype(np.float64) - out["reward"])
    assert (err <= tol).all(), f"reward: max err {err.max()} (tol {tol[err.argmax() // tol.shape[1]].max()})"
    if "logp" in rec:
        np.testing.assert_allclose(rec["logp"], out["logp"], rtol=TOL_F32, atol=1e-5)
    return out, st


def check_env_sites(w, rec_sites):
    """One-step checks at sampled (t, n) sites of a big rollout.

    rec_sites: dict of numpy arrays indexed by site i:
        obs [R, S] (before), obs_next [R, S], mu [R, D], noise [R, D], act_raw [R, D], shares [R, D],
        reward [R], done [R], tau [R] (cursor before the step), horizon (int),
        p0/i0 [R, D]/[R, DK] market row 0, p_now/i_now, p_val/i_val (rows tau and tau+1).
    Decodes cash and holdings exactly from the recorded observation (power-of-two scales)."""
    D, K = w.n_stocks, w.n_ind
    R = rec_sites["obs"].shape[0]
    obs = rec_sites["obs"]
    cash = (obs[:, 0] / np.float32(w.obs_scale[0])).astype(np.float32)
    hold = np.round(obs[:, 1 + D:1 + 2 * D].astype(np.float64) / w.obs_scale[2]).astype(np.int32)
    assert np.array_equal((hold.astype(np.float32) * np.float32(w.obs_scale[2])), obs[:, 1 + D:1 + 2 * D])
    done_site = (rec_sites["tau"] + 1) == rec_sites["horizon"]
    n_checked = 0
    for is_done in (False, True):
        sel = np.nonzero(done_site == is_done)[0]
        if sel.size == 0:
            continue
        # compact 3-row market per site: row 0 = the path's first row, row 1 = execution row, row 2 = valuation row
        # (a fourth row that the single step never reads keeps the table as long as the not-done horizon asks)
        price = np.stack([rec_sites["p0"][sel], rec_sites["p_now"][sel], rec_sites["p_val"][sel],
                          rec_sites["p_val"][sel]]).astype(np.float32)
        ind = np.stack([rec_sites["i0"][sel], rec_sites["i_now"][sel], rec_sites["i_val"][sel],
                        rec_sites["i_val"][sel]]).astype(np.float32)
        cfg = oracle.cfg_from_workload(w, horizon=2 if is_done else 3)
        st = oracle.State(cfg, sel.size)
        st.cash[:] = cash[sel]
        st.h[:] = hold[sel]
        st.tau[:] = 1
        for j, i in enumerate(sel):
            st.asset[j] = oracle.asset(float(cash[i]), hold[i], rec_sites["p_now"][i])
        out, st = oracle.rollout(cfg, w.hidden, bool(w.mlp_dtype), 1, price, ind, rec_sites["noise"][sel][None],
                                 mu_forced=rec_sites["mu"][sel][None], state=st,
                                 want=("obs", "act_raw", "reward", "done", "shares", "flags"))
        assert np.array_equal(out["act_raw"][0].view(np.uint32), rec_sites["act_raw"][sel].view(np.uint32))
        assert np.array_equal(out["shares"][0], rec_sites["shares"][sel]), "share counts"
        assert np.array_equal(out["done"][0], rec_sites["done"][sel]) and bool(out["done"][0].all()) == is_done
        assert np.array_equal(out["obs"][0].view(np.uint32), obs[sel].view(np.uint32)), "obs before"
        assert np.array_equal(out["obs"][1].view(np.uint32), rec_sites["obs_next"][sel].view(np.uint32)), "obs after"
        tol = reward_tolerance(w, out["reward"][0])
        assert (np.abs(rec_sites["reward"][sel].astype(np.float64) - out["reward"][0]) <= tol).all(), "reward"
        n_checked += sel.size
    assert n_checked == R
    return n_checked


def gae_tolerance(reward, value, done, gamma, lam):
    """Forward-error bound of the recurrence: 1e-4 * sum_l (gamma lam)^l |delta_{t+l}| (masked by episode ends)."""
    r = np.asarray(reward, np.float64)
    v = np.asarray(value, np.float64)
    nd = 1.0 - np.asarray(done, np.float64)
    delta = np.abs(r) + gamma * nd * np.abs(v[1:]) + np.abs(v[:-1])
    bound = np.zeros_like(delta)
    nxt = np.zeros(delta.shape[1])
    for t in range(delta.shape[0] - 1, -1, -1):
        nxt = delta[t] + gamma * lam * nd[t] * nxt
        bound[t] = nxt
    return TOL_F32 * bound


def check_gae(reward, value, done, gamma, lam, adv_gpu, ret_gpu):
    adv, ret = oracle.gae(reward, value, done, gamma, lam)
    tol = gae_tolerance(reward, value, done, gamma, lam)
    ea = np.abs(adv_gpu.astype(np.float64) - adv)
    er = np.abs(ret_gpu.astype(np.float64) - ret)
    assert (ea <= tol).all(), f"adv: worst ratio {(ea / tol).max()}"
    assert (er <= tol).all(), f"ret: worst ratio {(er / tol).max()}"
    return float((ea / tol).max())


def guard_cases(n, cost, seed=11):
    """(price, wanted-affordable count m, cash) triples at which the binary32 quotient cash / u rounds UP to the
    integer m although m shares cost more than the cash (u = fl(price * fl(1 + cost))): the purchase rule must then
    buy m - 1.  Built with exact rational arithmetic; returns float32 arrays p, cash and int array m, n of each."""
    from fractions import Fraction
    rng = np.random.default_rng(seed)
    one_plus_c = np.float32(np.float32(1.0) + np.float32(cost))
    ps, ms, cs = [], [], []
    while len(ps) < n:
        p = np.float32(rng.uniform(10, 100))
        u = np.float32(p * one_plus_c)
        m = int(rng.integers(2, 100))
        cash = np.float32(np.float32(m) * u)
        for _ in range(4):
            if Fraction(float(cash)) < m * Fraction(float(u)):
                break
            cash = np.nextafter(cash, np.float32(0))
        if Fraction(float(cash)) >= m * Fraction(float(u)) or np.float32(cash / u) != np.float32(m):
            continue
        if np.float32(np.float32(m) * u) > cash:      # the rounded outlay of m shares exceeds the cash: guard fires
            ps.append(p), ms.append(m), cs.append(cash)
    return np.array(ps, np.float32), np.array(ms, np.int64), np.array(cs, np.float32)
