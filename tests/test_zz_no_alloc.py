"""The entry point for callers that cannot allocate (scratch in a fixed device array inside the library) against
the workspace-taking entry point it is a variant of: same kernels, so the results must agree bit for bit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2112_05923_amd import inputs, podrollout as pr

DEV = "cuda:0"


def _case(w, B, R, seed):
    rng = np.random.default_rng(seed)
    S, D = w.state_dim, w.n_stocks
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)
    nets = {k: {kk: t(vv[0]) for kk, vv in inputs.make_weights(w, critic=(k == "critic")).items()}
            for k in ("actor", "critic")}
    obs = rng.standard_normal((R, S)).astype(np.float32)
    obs[:, 0] *= 0.5
    act = rng.uniform(-1.5, 1.5, (R, D)).astype(np.float32)
    logp_old = rng.normal(-30.0, 3.0, R).astype(np.float32)
    adv = rng.standard_normal(R).astype(np.float32)
    ret = rng.standard_normal(R).astype(np.float32)
    rows = torch.from_numpy(rng.permutation(R)[:B].astype(np.int32)).to(DEV)
    return nets, (t(obs), t(act), t(logp_old), t(adv), t(ret), rows)


def _empty_grads(cfg, fill):
    mk = lambda shapes: {k: torch.full(v, fill, dtype=torch.float32, device=DEV) for k, v in shapes.items()}
    return mk(pr._net_shapes(cfg, cfg.n_stocks)), mk(pr._net_shapes(cfg, 1))


@pytest.mark.gpu
def test_noalloc_minibatch_grads_equal_the_workspace_entry_point_on_two_calls_in_a_row():
    # the paper's minibatch on the headline network shape first, a smaller batch on a smaller network second:
    # the second call finds the first call's contents in the shared scratch
    for name, B, R in (("large", 1024, 1300), ("dow30", 96, 200)):
        w = inputs.WORKLOADS[name]
        cfg = pr.make_ppo_config(w, batch=B)
        nets, batch = _case(w, B, R, seed=B)
        want_a, want_c, want_stats = pr.ppo_minibatch_grads(cfg, *batch, nets["actor"], nets["critic"])
        ga, gc = _empty_grads(cfg, float("nan"))
        stats = torch.full((4,), float("nan"), device=DEV)
        pr.ppo_minibatch_grads_noalloc(cfg, *batch, nets["actor"], nets["critic"], ga, gc, stats)
        torch.cuda.synchronize()
        for k in pr.NET_KEYS:
            assert torch.equal(ga[k], want_a[k]), (name, "actor", k)
            assert torch.equal(gc[k], want_c[k]), (name, "critic", k)
        assert torch.equal(stats, want_stats), name
        assert bool(torch.isfinite(ga["W1"]).all()) and float(ga["W2"].abs().max()) > 0.0


@pytest.mark.gpu
def test_noalloc_refuses_shapes_beyond_its_scratch_and_bad_arguments():
    w = inputs.WORKLOADS["large"]
    cfg = pr.make_ppo_config(w, batch=4096)          # 4x the scratch of the 1024-row minibatch
    n = C.c_size_t(0)
    assert pr.lib().ppo_workspace_bytes(C.byref(cfg), C.byref(n)) == pr.PR_OK and n.value > pr.PR_STATIC_SCRATCH_BYTES
    nets, batch = _case(w, 4096, 4096, seed=1)
    ga, gc = _empty_grads(cfg, 7.0)
    stats = torch.zeros(4, device=DEV)
    with pytest.raises(pr.PodError) as e:
        pr.ppo_minibatch_grads_noalloc(cfg, *batch, nets["actor"], nets["critic"], ga, gc, stats)
    assert e.value.code == pr.PR_ETOOBIG and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(ga["W1"].min()) == 7.0 and float(ga["W1"].max()) == 7.0       # nothing was enqueued
    assert pr.lib().ppo_minibatch_grads_noalloc(None, C.byref(cfg), *([None] * 6), *([None] * 4), None) == pr.PR_EINVAL
