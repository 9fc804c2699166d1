"""Pins of the checker's PPO minibatch (Sec. 4.2 learner; Sec. 5.2: PPO, batch 1024, lr 1e-3) and Adam: finite
differences of the loss, the hand-derivable cases of the clipped surrogate, closed forms of the first Adam step."""
import numpy as np
import pytest

import oracle

S, HD, D = 9, 8, 3
SIGMA, CLIP, CV = 0.5, 0.2, 0.5


def _nets(rng, scale=0.4):
    shp = {"W1": (S, HD), "b1": (HD,), "W2": (HD, HD), "b2": (HD,)}
    a = {k: (scale * rng.standard_normal(v)).astype(np.float32) for k, v in shp.items()}
    c = {k: (scale * rng.standard_normal(v)).astype(np.float32) for k, v in shp.items()}
    a["W3"], a["b3"] = (scale * rng.standard_normal((HD, D))).astype(np.float32), (scale * rng.standard_normal(D)).astype(np.float32)
    c["W3"], c["b3"] = (scale * rng.standard_normal((HD, 1))).astype(np.float32), (scale * rng.standard_normal(1)).astype(np.float32)
    return a, c


def _mlp(x, n, out_tanh):
    h = np.tanh(x @ n["W1"].astype(np.float64) + n["b1"])
    h = np.tanh(h @ n["W2"].astype(np.float64) + n["b2"])
    z = h @ n["W3"].astype(np.float64) + n["b3"]
    return np.tanh(z) if out_tanh else z


def _loss(obs, act, logp_old, adv, ret, a, c):
    """The objective written with numpy (no gradients): what the checker's gradients must be the slope of."""
    mu = _mlp(obs.astype(np.float64), a, True)
    v = _mlp(obs.astype(np.float64), c, False)[:, 0]
    logp = (-(act - mu) ** 2 / (2 * SIGMA ** 2)).sum(1) - D * np.log(SIGMA) - 0.5 * D * np.log(2 * np.pi)
    ratio = np.exp(logp - logp_old)
    l_pi = -np.minimum(ratio * adv, np.clip(ratio, 1 - CLIP, 1 + CLIP) * adv).mean()
    l_v = 0.5 * ((v - ret) ** 2).mean()
    return l_pi + CV * l_v, l_pi, l_v, ratio


def _batch(rng, B, a):
    obs = rng.standard_normal((B, S)).astype(np.float32)
    mu = _mlp(obs.astype(np.float64), a, True)
    act = (mu + SIGMA * rng.standard_normal((B, D))).astype(np.float32)
    logp = (-(act - mu) ** 2 / (2 * SIGMA ** 2)).sum(1) - D * np.log(SIGMA) - 0.5 * D * np.log(2 * np.pi)
    # old log-probs scattered around the new ones so that ratios fall inside and outside the clip range
    logp_old = (logp + rng.normal(0, 0.25, B)).astype(np.float32)
    adv = rng.standard_normal(B).astype(np.float32)
    ret = rng.standard_normal(B).astype(np.float32)
    return obs, act, logp_old, adv, ret


def test_loss_values_and_statistics_match_the_numpy_objective():
    rng = np.random.default_rng(0)
    a, c = _nets(rng)
    batch = _batch(rng, 64, a)
    _, _, stats, margin = oracle.ppo_grads(*batch, a, c, SIGMA, CLIP, CV)
    total, l_pi, l_v, ratio = _loss(*batch, a, c)
    assert stats[0] == pytest.approx(l_pi, rel=1e-12) and stats[1] == pytest.approx(l_v, rel=1e-12)
    cut = (ratio * batch[3]) > (np.clip(ratio, 1 - CLIP, 1 + CLIP) * batch[3])
    assert stats[2] == pytest.approx(cut.mean()) and 0.1 < cut.mean() < 0.9     # both branches are exercised
    assert stats[3] == pytest.approx(ratio.mean(), rel=1e-12)
    np.testing.assert_allclose(margin, np.minimum(abs(ratio - (1 - CLIP)), abs(ratio - (1 + CLIP))), rtol=1e-9)


def test_gradients_are_the_slope_of_the_objective():
    rng = np.random.default_rng(1)
    a, c = _nets(rng)
    batch = _batch(rng, 48, a)
    ga, gc, _, margin = oracle.ppo_grads(*batch, a, c, SIGMA, CLIP, CV)
    assert margin.min() > 1e-4        # no sample sits on a kink of min / clip
    for net, g, which in ((a, ga, "a"), (c, gc, "c")):
        for k in oracle.NET_KEYS:
            flat = net[k].reshape(-1)
            for i in rng.choice(flat.size, size=min(6, flat.size), replace=False):
                old = flat[i]
                h = np.float32(2.0 ** -13)        # exactly representable steps around an fp32 weight
                flat[i] = old + h
                up = _loss(*batch, a, c)[0]
                flat[i] = old - h
                dn = _loss(*batch, a, c)[0]
                flat[i] = old
                fd = (up - dn) / (2.0 * float(h))
                assert g[k].reshape(-1)[i] == pytest.approx(fd, rel=2e-5, abs=1e-9), (which, k, i)


def test_clipped_surrogate_cases():
    rng = np.random.default_rng(2)
    a, c = _nets(rng)
    obs, act, logp_old, adv, ret = _batch(rng, 8, a)
    mu = _mlp(obs.astype(np.float64), a, True)
    logp = (-(act - mu) ** 2 / (2 * SIGMA ** 2)).sum(1) - D * np.log(SIGMA) - 0.5 * D * np.log(2 * np.pi)
    # ratio 1.5 with positive advantage and ratio 0.5 with negative advantage: the minimum cuts, no policy gradient
    lo = np.where(np.arange(8) % 2 == 0, logp - np.log(1.5), logp - np.log(0.5)).astype(np.float32)
    ad = np.where(np.arange(8) % 2 == 0, 1.0, -1.0).astype(np.float32)
    ga, _, stats, _ = oracle.ppo_grads(obs, act, lo, ad, ret, a, c, SIGMA, CLIP, CV)
    assert stats[2] == 1.0 and all(np.all(ga[k] == 0.0) for k in oracle.NET_KEYS)
    assert stats[0] == pytest.approx(-np.mean(np.where(ad > 0, 1 + CLIP, -(1 - CLIP))), rel=1e-6)
    # the same ratios with the advantages swapped: outside the range on the side the minimum keeps -> gradient flows
    ga, _, stats, _ = oracle.ppo_grads(obs, act, lo, -ad, ret, a, c, SIGMA, CLIP, CV)
    assert stats[2] == 0.0 and any(np.any(ga[k] != 0.0) for k in oracle.NET_KEYS)
    # ratio exactly 1: the policy gradient is that of -A logp / B
    ga, gc, stats, _ = oracle.ppo_grads(obs, act, logp.astype(np.float32), adv, ret, a, c, SIGMA, CLIP, CV)
    e = act - mu
    dz3 = -(adv[:, None] * np.exp(logp - logp.astype(np.float32))[:, None] * e / SIGMA ** 2) / 8 * (1 - mu ** 2)
    np.testing.assert_allclose(ga["b3"], dz3.sum(0), rtol=1e-9)
    # the critic's gradient does not depend on the policy terms and scales with the value coefficient
    _, gc2, _, _ = oracle.ppo_grads(obs, act, lo, ad, ret, a, c, SIGMA, CLIP, 2 * CV)
    for k in oracle.NET_KEYS:
        np.testing.assert_allclose(gc2[k], 2.0 * gc[k], rtol=1e-12)
    v = _mlp(obs.astype(np.float64), c, False)[:, 0]
    assert gc["b3"][0] == pytest.approx(CV * np.mean(v - ret), rel=1e-9)


def test_adam_first_step_and_recurrence():
    rng = np.random.default_rng(4)
    g = rng.standard_normal(33)
    th0 = rng.standard_normal(33)
    th, m, v = oracle.adam(th0, g, np.zeros(33), np.zeros(33), 1e-3, 0.9, 0.999, 1e-8, 1)
    # with zero moments the bias-corrected first step is lr * g / (|g| + eps): lr in size, against the gradient
    np.testing.assert_allclose(th0 - th, 1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-9)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-9)
    # three steps against the recurrence written with numpy
    tm, mm, vm = th0.copy(), np.zeros(33), np.zeros(33)
    to, mo, vo = th0.copy(), np.zeros(33), np.zeros(33)
    for t in (1, 2, 3):
        gt = rng.standard_normal(33)
        mm = 0.9 * mm + 0.1 * gt
        vm = 0.999 * vm + 0.001 * gt ** 2
        tm = tm - 1e-3 * (mm / (1 - 0.9 ** t)) / (np.sqrt(vm / (1 - 0.999 ** t)) + 1e-8)
        to, mo, vo = oracle.adam(to, gt, mo, vo, 1e-3, 0.9, 0.999, 1e-8, t)
    np.testing.assert_allclose(to, tm, rtol=1e-12)
