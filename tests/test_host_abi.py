"""Host-only checks of the C-ABI library: it loads, exports every function the
header declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2112_05923_amd import inputs, podrollout as pr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "podrollout.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"^\s*(?:int|const char \*)\s*\**(\w+)\s*\(", src, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_entry_point():
    names = _declared()
    assert {"rollout_init", "rollout_step_T", "compute_gae"} <= set(names)
    assert sorted(pr.EXPORTS) == names
    lib = pr.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_header_layout():
    assert C.sizeof(pr.PrConfig) == 9 * 4 + 5 * 4 + 4 * 4
    assert C.sizeof(pr.PrBuffers) == 8 * 8 and C.sizeof(pr.PrState) == 7 * 8 and C.sizeof(pr.PrWeights) == 6 * 8


def test_strerror():
    lib = pr.lib()
    assert lib.rollout_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert lib.rollout_strerror(code)


def _ws(cfg):
    n = C.c_size_t(0)
    return pr.lib().rollout_workspace_bytes(C.byref(cfg), C.byref(n)), n.value


def test_workspace_query_and_config_validation():
    w = inputs.WORKLOADS["large"]
    rc, n = _ws(pr.make_config(w))
    assert rc == pr.PR_OK and n > 16384 * 30 * 8
    for name in inputs.WORKLOADS:
        rc, n = _ws(pr.make_config(inputs.WORKLOADS[name]))
        assert rc == pr.PR_OK, name
    bad = [dict(n_envs=0), dict(n_agents=3), dict(n_stocks=0), dict(n_ind=-1), dict(horizon=0), dict(n_market=7),
           dict(mlp_dtype=2), dict(schedule=5), dict(cash0=0.0), dict(hmax=-1.0), dict(cost=1.0), dict(cost=-0.1),
           dict(sigma=0.0)]
    for kw in bad:
        cfg = pr.make_config(w)
        for k, v in kw.items():
            setattr(cfg, k, v)
        rc, _ = _ws(cfg)
        assert rc == pr.PR_EINVAL, kw
    cfg = pr.make_config(w)
    cfg.obs_scale[1] = 0.3          # not a power of two
    assert _ws(cfg)[0] == pr.PR_EINVAL
    cfg = pr.make_config(w)
    cfg.hidden = 100                # not a multiple of 32
    assert _ws(cfg)[0] == pr.PR_EUNSUPPORTED
    cfg = pr.make_config(w.replace(n_agents=16384 // 32))   # 32 envs per agent: tiles would straddle agents
    assert _ws(cfg)[0] == pr.PR_EUNSUPPORTED
    assert pr.lib().rollout_workspace_bytes(None, None) == pr.PR_EINVAL


def test_persistent_kernel_lds_fits_the_compute_unit_for_every_shape_it_accepts():
    """The launch of the persistent kernel takes its LDS size from the same carve-up this query reads; every
    shape the schedule accepts must fit the 160 KiB of a compute unit, with and without the actor, and the
    schedule must accept the named workloads it is documented for."""
    limit = 160 * 1024
    seen = 0
    for dtype, hiddens in ((1, (256, 512)), (0, (256,))):
        for hidden in hiddens:
            for D in (1, 2, 5, 17, 24, 30, 32):
                for K in (1, 2, 4, 7, 8, 10, 16):
                    w = inputs.WORKLOADS["large"].replace(n_envs=128, n_stocks=D, n_ind=K, hidden=hidden, mlp_dtype=dtype)
                    cfg = pr.make_config(w, horizon=8, schedule=pr.PR_SCHED_FUSED)
                    try:
                        a, b = pr.kernel_lds_bytes(cfg, True), pr.kernel_lds_bytes(cfg, False)
                    except pr.PodError as e:
                        assert e.code == pr.PR_EUNSUPPORTED
                        continue
                    seen += 1
                    assert 0 < b <= a <= limit, (dtype, hidden, D, K, a, b)
    assert seen >= 40
    for name in ("large", "dow30", "tournament"):
        cfg = pr.make_config(inputs.WORKLOADS[name], schedule=pr.PR_SCHED_FUSED)
        assert pr.kernel_lds_bytes(cfg) <= limit
    for name in ("wide",):   # 500 stocks: per-step schedule only
        with pytest.raises(pr.PodError):
            pr.kernel_lds_bytes(pr.make_config(inputs.WORKLOADS[name], schedule=pr.PR_SCHED_FUSED))


def test_null_arguments_are_rejected_without_device_work():
    lib = pr.lib()
    cfg = pr.make_config(inputs.WORKLOADS["tiny"])
    h = C.c_void_p()
    m, wa = pr.PrMarket(), pr.PrWeights()
    assert lib.rollout_init(C.byref(cfg), C.byref(m), C.byref(wa), C.byref(wa), None, 0, None, C.byref(h)) == pr.PR_EINVAL
    assert not h.value
    assert lib.rollout_init(C.byref(cfg), None, None, None, None, 0, None, None) == pr.PR_EINVAL
    assert lib.rollout_step_T(None, 4, None, None) == pr.PR_EINVAL
    assert lib.rollout_step_forced(None, 4, None, None, None) == pr.PR_EINVAL
    assert lib.rollout_mlp_forward(None, 0, 1, None, 1, None) == pr.PR_EINVAL
    assert lib.rollout_reset(None) == pr.PR_EINVAL
    assert lib.rollout_set_replay(None, None, 0, None) == pr.PR_EINVAL
    assert lib.rollout_destroy(None) == pr.PR_EINVAL
    assert lib.rollout_leaderboard(None, None, None, None) == pr.PR_EINVAL
    assert lib.compute_gae(None, 0, 4, None, None, None, 0.99, 0.95, None, None) == pr.PR_EINVAL
    assert lib.compute_gae(None, 4, 4, None, None, None, 0.99, 0.95, None, None) == pr.PR_EINVAL
    assert lib.trading_metrics(None, 4, 4, 3, 13, None, None, None, 252.0, 0.0, None, None) == pr.PR_EINVAL
    assert lib.population_refill(None, 4, 16, None, 2, 0.0, None, None) == pr.PR_EINVAL
    cfg = pr.PrPpoConfig(1024, 30, 8, 512, 0.5, 0.2, 0.5, 1e-3, 0.9, 0.999, 1e-8, 1)
    n = C.c_size_t(0)
    assert lib.ppo_workspace_bytes(C.byref(cfg), C.byref(n)) == pr.PR_OK and n.value > 4 * 1024 * 512 * 4
    bad = pr.PrPpoConfig(1024, 30, 8, 500, 0.5, 0.2, 0.5, 1e-3, 0.9, 0.999, 1e-8, 1)
    assert lib.ppo_workspace_bytes(C.byref(bad), C.byref(n)) == pr.PR_EINVAL
    assert lib.adam_update(None, 0, None, None, None, None, 1e-3, 0.9, 0.999, 1e-8, 1) == pr.PR_EINVAL
    assert lib.ppo_minibatch_grads(None, C.byref(cfg), *([None] * 6), *([None] * 4), None, 0, None) == pr.PR_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(pr, "_lib", None)
    monkeypatch.setattr(pr, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libpodrollout.so"))
    with pytest.raises(FileNotFoundError):
        pr.lib()


def test_bench_refuses_more_than_one_gpu_and_reads_the_recorded_traffic():
    """bench.py is a one-GPU benchmark: --gpus 2 must exit with a message before touching a device.  The traffic
    figure it reports is the recorded one only while the kernel sources still hash to the recorded digest."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.kernel_sources_digest()
    assert re.fullmatch(r"[0-9a-f]{16}", digest)
    text = open(os.path.join(ROOT, "profiles", "pmc_fused_large.txt")).read()
    recorded = re.search(r"kernel_sources_digest: (\w+)", text).group(1)
    got = bench.recorded_traffic("fused", "large")
    if recorded == digest:
        assert got == pytest.approx(float(re.search(r"hbm_bytes_per_launch: (\d+)", text).group(1)))
    else:
        assert got is None
