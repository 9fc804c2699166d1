"""Stage-wise comparison of a GPU rollout record with the CPU checker.

The map from the policy mean to the trajectory is discontinuous (share counts
are truncated), so stages are compared with their inputs taken from the GPU's
own record: the networks on the recorded observations, the environment on the
recorded means and noise.

Tolerances.  Integers and everything that is an exact function of them are
compared bit for bit.  Network outputs: 1e-4 relative (fp32 operands), 2e-2
relative (bf16 operands), where "relative" is to the size of the output vector
the value belongs to (the largest |entry| of the row for the actor; of the
compared batch for the scalar critic).  An entry-wise relative error is not
meaningful for entries near zero: binary32 accumulation over 301 + 256 terms
leaves an absolute error of about 2e-6 on outputs of size 1 whatever the
entry, and with bf16 activations a single one-ulp re-quantisation flip in the
first hidden layer moves every output by up to about 5e-3 (measured on 65 536
rows: 2.2e-6 and 5.2e-3 of the row maximum).
"""
from __future__ import annotations

import numpy as np

import oracle

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def to_np(t):
    return t.detach().cpu().numpy()


def rel_err_rows(got, want):
    """max |got - want| / (largest |want| of the same row), rows = last axis."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    scale = np.maximum(np.abs(want).max(axis=-1, keepdims=True), 1e-30)
    return float((np.abs(got - want) / scale).max())


def check_networks(w, weights_actor, weights_critic, obs_rows, mu_rows=None, value_rows=None, agent=0):
    """obs_rows [R, S] from the GPU record -> checker outputs vs recorded mu / value of the same rows."""
    tol = TOL_BF16 if w.mlp_dtype else TOL_F32
    errs = {}
    if mu_rows is not None:
        a = {k: v[agent] for k, v in weights_actor.items()}
        want = oracle.mlp(obs_rows, a["W1"], a["b1"], a["W2"], a["b2"], a["W3"], a["b3"], True, bool(w.mlp_dtype))
        errs["mu"] = rel_err_rows(mu_rows, want)
        assert errs["mu"] <= tol, errs
    if value_rows is not None:
        c = {k: v[agent] for k, v in weights_critic.items()}
        want = oracle.mlp(obs_rows, c["W1"], c["b1"], c["W2"], c["b2"], c["W3"], c["b3"], False, bool(w.mlp_dtype))
        # the critic has one output per row: scale by the size of the values in the batch
        got = np.asarray(value_rows, np.float64).reshape(-1)
        want = want.reshape(-1)
        errs["value"] = float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))
        assert errs["value"] <= tol, errs
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
