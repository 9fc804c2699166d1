#!/usr/bin/env python3
"""Throughput of the whole rollout hot path on one MI355X.

One "step" = one pass of the path over one batch of synthetic input: T steps of
{actor forward, Gaussian sampling, trading-env step} for N envs, the critic on
all T+1 observations, and GAE -- the three C-ABI calls rollout_step_T (without
values), rollout_mlp_forward (critic on the whole observation buffer, the same
launch rollout_step_T makes when given a value buffer) and compute_gae, issued
back to back with HIP events between them so that each stage is timed inside
the timed region.  Inputs are resident in HBM before the clock starts.

Prints ONE JSON line (metric env-steps/s) with a roofline object for the
dominant kernel and the CPU checker's rate on the host cores.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm": (8000.0, "GB/s"), "mfma_bf16": (2500.0, "TFLOP/s"), "mfma_fp32": (157.3, "TFLOP/s")}


def kernel_sources_digest() -> str:
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2112_05923_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed counter summary, or None when the
    kernel sources changed after the counters were taken."""
    path = os.path.join(ROOT, "profiles", f"pmc_{kernel}_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    if vals.get("kernel_sources_digest") != kernel_sources_digest():
        return None
    try:
        return float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def cpu_baseline(w, n_envs: int, steps: int, threads: int):
    """The CPU checker as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2112_05923_amd import inputs

    ws = w.replace(n_envs=n_envs, steps=steps)
    d = inputs.make_all(ws)
    cfg = oracle.cfg_from_workload(ws)
    chunks = np.array_split(np.arange(n_envs), threads)

    def work(idx):
        if idx.size == 0:
            return 0
        out, _ = oracle.rollout(cfg, ws.hidden, bool(ws.mlp_dtype), steps, d["price"][:, idx], d["ind"][:, idx],
                                d["noise"][:, idx], actor=d["actor"], critic=d["critic"],
                                want=("obs", "act_raw", "logp", "reward", "done", "value"))
        oracle.gae(out["reward"], out["value"], out["done"], ws.gamma, ws.lam)
        return idx.size

    oracle.lib()
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=threads) as ex:
        done = sum(ex.map(work, chunks))
    dt = time.perf_counter() - t0
    # the same code on one core, on a smaller slice of the same sample
    one = np.arange(max(1, n_envs // threads))
    t1 = time.perf_counter()
    work(one)
    dt1 = time.perf_counter() - t1
    return {"value": done * steps / dt, "unit": "env-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_envs} envs x {steps} steps of workload '{w.name}' (free-running rollout + critic + GAE), "
                      f"{dt:.1f} s wall",
            "one_core": {"value": one.size * steps / dt1, "unit": "env-steps/s",
                         "sample": f"{one.size} envs x {steps} steps, {dt1:.1f} s wall"}}


def side_measurements(torch, pr, inputs, w, d, out, roll, adv, ret, obs2d, val2d, sched, dev):
    """Untimed companions of the path, measured on the record the timed steps just produced; none of them is part
    of `value`."""
    T, N, D = w.steps, w.n_envs, w.n_stocks
    env_steps = N * T
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # the evaluator's trading figures
    pr.trading_metrics(out["obs"], out["done"], D, w.obs_scale, 252.0 * 390.0)
    e0.record()
    for _ in range(3):
        pr.trading_metrics(out["obs"], out["done"], D, w.obs_scale, 252.0 * 390.0)
    e1.record()
    torch.cuda.synchronize()
    t_metrics = e0.elapsed_time(e1) / 3

    # (also outside) the generator step on a 64-agent block of 512 x 512 weights, 16 candidates kept
    pop = torch.randn((64, 512, 512), device=dev)
    pop_noise = torch.randn((64, 512, 512), device=dev)
    pop_rank = torch.randperm(64, device=dev).to(torch.int32)
    pr.population_refill(pop, pop_rank, 16, 0.02, pop_noise)
    e0.record()
    for _ in range(10):
        pr.population_refill(pop, pop_rank, 16, 0.02, pop_noise)
    e1.record()
    torch.cuda.synchronize()
    t_pop = e0.elapsed_time(e1) / 10
    del pop, pop_noise

    # (also outside) one PPO minibatch step of the learner (Sec. 5.2: batch 1024) on rows drawn from this buffer
    t_learn = None
    if w.n_agents == 1:
        lcfg = pr.make_ppo_config(w, batch=1024)
        host_nets = {k: inputs.make_weights(w, critic=(k == "critic")) for k in ("actor", "critic")}
        nets = {k: {kk: torch.from_numpy(vv[0]).to(dev) for kk, vv in n.items()} for k, n in host_nets.items()}
        zeros = lambda n: {k: torch.zeros_like(v) for k, v in n.items()}
        mom = [zeros(nets["actor"]), zeros(nets["actor"]), zeros(nets["critic"]), zeros(nets["critic"])]
        lws = pr.ppo_workspace(lcfg, dev)
        g = torch.Generator(device=dev)
        g.manual_seed(inputs.BASE_SEED)
        rows = torch.randint(0, T * N, (1024,), generator=g, device=dev, dtype=torch.int32)
        learn = lambda: pr.ppo_learner_step(lcfg, obs2d[:T * N], out["act_raw"].view(T * N, D), out["logp"].view(-1),
                                            adv.view(-1), ret.view(-1), rows, nets["actor"], nets["critic"], *mom, lws)
        learn()
        e0.record()
        for _ in range(10):
            learn()
        e1.record()
        torch.cuda.synchronize()
        t_learn = e0.elapsed_time(e1) / 10

    # (also outside) the same step on one shared market table of 2^17 rows replayed from random per-env start rows,
    # cost 0.2 % (Sec. 5.3 set-up: every env trades the same minute-level data set)
    t_replay = None
    if w.n_agents == 1:
        R = 1 << 17
        wr = w.replace(cost=2.0e-3)
        tab = inputs.make_all_device(wr, dev, horizon=R - 1, n_market=1, steps=1)
        ro2 = pr.Rollout(pr.make_config(wr, horizon=T, n_market=1, schedule=sched), tab["price"][:T + 1],
                         tab["ind"][:T + 1], d["actor"], d["critic"])
        g = torch.Generator(device=dev)
        g.manual_seed(inputs.BASE_SEED + 1)
        ro2.set_replay(tab["price"], tab["ind"],
                       torch.randint(0, R - T, (N,), generator=g, device=dev, dtype=torch.int32))

        def replay_step():
            ro2.reset()
            ro2.step_T(T, d["noise"], roll)
            ro2.mlp_forward(pr.PR_NET_CRITIC, obs2d, val2d)
            pr.compute_gae(out["reward"], out["value"], out["done"], w.gamma, w.lam, adv, ret)

        replay_step()
        e0.record()
        for _ in range(3):
            replay_step()
        e1.record()
        torch.cuda.synchronize()
        t_replay = e0.elapsed_time(e1) / 3
        ro2.close()
        del tab

    extras = {"trading_metrics": {"ms": t_metrics, "note": "not part of value; reads 4(1+2D) of every 4S-byte row",
                                  "GBps": (4 * (1 + 2 * D) + 1) * (T + 1) * N / t_metrics / 1e6},
              "population_refill": {"ms": t_pop, "note": "not part of value; 48 of 64 agents x 512 x 512 weights, "
                                                         "12 B per rewritten weight",
                                    "GBps": 48 * 512 * 512 * 12 / t_pop / 1e6}}
    if t_learn is not None:
        extras["ppo_learner_step"] = {"ms": t_learn, "samples_per_s": 1024 / t_learn * 1e3,
                                      "note": "not part of value; minibatch 1024 gathered from this buffer, both "
                                              "networks forward + backward + Adam, fp32, eager launches"}
    if t_replay is not None:
        extras["replay_shared_table"] = {"ms": t_replay, "env_steps_per_s": env_steps / t_replay * 1e3,
                                         "note": "not part of value; the same step with M = 1, a table of 131072 "
                                                 "rows, random per-env start rows, cost 0.2 %"}
    return extras


def measured_peaks():
    """Two short launches that say what this machine delivers where the roofline uses published figures: the matrix
    pipe alone (bf16, two wavefronts per SIMD of independent matrix instructions) and a streaming read of 1 GiB."""
    import torch
    from paper_2112_05923_amd import podrollout as pr

    dev = torch.device("cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    sink = torch.empty(64, dtype=torch.float32, device=dev)
    pr.calibrate_stream(pr.PR_CAL_READ, src, sink)
    torch.cuda.synchronize()
    e0.record()
    pr.calibrate_stream(pr.PR_CAL_READ, src, sink)
    e1.record()
    torch.cuda.synchronize()
    read_gbps = src.numel() * 4 / e0.elapsed_time(e1) / 1e6
    del src
    IM = 4096
    ticks = torch.full((256, 8), -1, dtype=torch.int64, device=dev)
    roles = [pr.ROLE_MATRIX] * 8
    pr.calibrate_probe(roles, IM, 0, 0, False, 256, ticks)
    pr.calibrate_probe(roles, IM, 0, 0, False, 256, ticks)
    torch.cuda.synchronize()
    t_us = float(ticks.cpu().numpy().astype("float64").mean() * 10.0 / 1e3)
    mfma_tflops = IM * 8 * 2 * 32 * 32 * 16 * 8 * 256 / (t_us * 1e-6) / 1e12
    return {"hbm_read_GBps": read_gbps, "mfma_bf16_TFLOPs": mfma_tflops,
            "note": "this box, measured in this run: streaming read of 1 GiB; 8 wavefronts per compute unit of "
                    "independent v_mfma_f32_32x32x16_bf16"}


def calibrate():
    """Measured machine figures the roofline fractions can be read against: streaming copy and read bandwidth,
    the matrix pipe alone, and how matrix instructions share a SIMD with the vector / transcendental
    instructions of a tanh epilogue (issued by another wavefront of the SIMD, or interleaved in one wavefront).
    Prints one JSON line; every entry is one launch timed with events (after one untimed launch)."""
    import torch
    from paper_2112_05923_amd import podrollout as pr

    dev = torch.device("cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    res = {}
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
    dst = torch.empty_like(src)
    nbytes = src.numel() * 4
    ms = timed(lambda: pr.calibrate_stream(pr.PR_CAL_COPY, src, dst))
    res["copy"] = {"GiB": 1, "ms": ms, "GBps_read_plus_write": 2 * nbytes / ms / 1e6}
    ms = timed(lambda: pr.calibrate_stream(pr.PR_CAL_READ, src, dst))
    res["read"] = {"GiB": 1, "ms": ms, "GBps": nbytes / ms / 1e6}
    del src, dst

    M, V, B, P, O = pr.ROLE_MATRIX, pr.ROLE_VECTOR, pr.ROLE_BOTH, pr.ROLE_PLAIN, pr.ROLE_NONE
    IM, IV = 4096, 1024           # 32768 matrix instructions / 32768 activations per lane and wavefront
    flop_per_wave = IM * 8 * 2 * 32 * 32 * 16
    cases = {
        "matrix_1_per_simd": ([M, M, M, M, O, O, O, O], 0, False),
        "matrix_2_per_simd": ([M] * 8, 0, False),
        "matrix_2_per_simd_lds_operand": ([M] * 8, 0, True),
        "vector_1_per_simd": ([V, V, V, V, O, O, O, O], 0, False),
        "vector_2_per_simd": ([V] * 8, 0, False),
        "plain_1_per_simd": ([P, P, P, P, O, O, O, O], 0, False),
        "plain_2_per_simd": ([P] * 8, 0, False),
        "matrix_and_vector_wavefronts_share_simd": ([M, M, M, M, V, V, V, V], 0, False),
        "matrix_lds_and_vector_wavefronts_share_simd": ([M, M, M, M, V, V, V, V], 0, True),
        "matrix_and_plain_wavefronts_share_simd": ([M, M, M, M, P, P, P, P], 0, False),
        "one_wavefront_both_2_acts_per_8": ([B, B, B, B, O, O, O, O], 2, False),
        "one_wavefront_both_4_acts_per_8": ([B, B, B, B, O, O, O, O], 4, False),
        "one_wavefront_both_8_acts_per_8": ([B, B, B, B, O, O, O, O], 8, False),
        "two_wavefronts_both_4_acts_per_8": ([B] * 8, 4, False),
        "two_wavefronts_both_8_acts_per_8": ([B] * 8, 8, False),
    }
    probes = {}
    for name, (roles, acts, lds) in cases.items():
        ticks = torch.full((256, 8), -1, dtype=torch.int64, device=dev)
        ms = timed(lambda: pr.calibrate_probe(roles, IM, IV, acts, lds, 256, ticks), reps=2)
        t = ticks.cpu().numpy().astype("float64") * 10.0      # ns per wavefront
        entry = {"launch_ms": ms}
        for role, label in ((M, "matrix"), (V, "vector"), (B, "both"), (P, "plain")):
            cols = [i for i, r in enumerate(roles) if r == role]
            if cols:
                entry[label + "_wavefront_us"] = float(t[:, cols].mean() / 1e3)
        n_m = sum(1 for r in roles if r in (M, B))
        if n_m:
            tm = entry.get("matrix_wavefront_us", entry.get("both_wavefront_us"))
            entry["matrix_TFLOPs_chip"] = flop_per_wave * n_m * 256 / (tm * 1e-6) / 1e12
            entry["ns_per_matrix_instruction_per_simd"] = tm * 1e3 / (IM * 8) / max(1, n_m // 4)
        n_v = sum(1 for r in roles if r in (V, P))
        if n_v:
            tv = entry.get("vector_wavefront_us", entry.get("plain_wavefront_us"))
            entry["ns_per_activation_per_simd"] = tv * 1e3 / (IV * 32) / max(1, n_v // 4)
        if acts:
            entry["activations_per_matrix_instruction"] = acts / 8
        probes[name] = entry
    res["probes"] = probes
    res["note"] = ("probe wavefronts: matrix = 32768 independent v_mfma_f32_32x32x16_bf16 each; vector = 32768 "
                   "activations (fma, exp2, add, rcp, fma) per lane each; both = the matrix loop with that many "
                   "activations interleaved in program order; 256 workgroups, one per compute unit")
    print(json.dumps({"calibration": res}))


def stages_alone(torch, pr, inputs, w, d, ro, out, roll, obs2d, sched, dev):
    """Each stage of the path launched on its own (untimed companions of the timed path; none is part of `value`):
    the environment + sampling stage with caller-supplied means (rollout_step_forced: the rollout's own kernel
    without the actor) and the actor on all T x N recorded observations in one launch (rollout_mlp_forward).  In
    the persistent schedule both live in one kernel, so these launches are what separates the environment's share
    of the HBM roofline from the actor's share of the matrix roofline."""
    T, N, D, S = w.steps, w.n_envs, w.n_stocks, w.state_dim
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    res = {}
    mf = "mfma_bf16" if w.mlp_dtype else "mfma_fp32"
    # actor over the recorded buffer
    mu = torch.empty((T * N, D), dtype=torch.float32, device=dev)
    ro.mlp_forward(pr.PR_NET_ACTOR, obs2d[:T * N], mu)
    e0.record()
    for _ in range(2):
        ro.mlp_forward(pr.PR_NET_ACTOR, obs2d[:T * N], mu)
    e1.record()
    torch.cuda.synchronize()
    t_actor = e0.elapsed_time(e1) / 2
    fl = inputs.mlp_flops_per_env_step(w, critic=False) * T * N
    res["actor_alone"] = {"ms": t_actor, "TFLOPs": fl / t_actor / 1e9, "frac_mfma": fl / t_actor / 1e9 / PEAK[mf][0],
                          "note": "rollout_mlp_forward(actor) on the T x N recorded observations, one launch"}
    # environment + sampling stage, forced onto the recorded means
    mu3 = mu.view(T, N, D)

    def forced():
        ro.reset()
        ro.step_forced(T, mu3, d["noise"], roll)

    forced()
    e0.record()
    for _ in range(2):
        forced()
    e1.record()
    torch.cuda.synchronize()
    t_env = e0.elapsed_time(e1) / 2
    by = inputs.bytes_per_env_step(w) * T * N
    res["env_alone"] = {"ms": t_env, "algorithmic_GBps": by / t_env / 1e6, "frac_hbm": by / t_env / 1e6 / PEAK["hbm"][0],
                        "note": "rollout_step_forced over T steps (observation assembly, sampling, trades, reward, "
                                "done / reset) with the means of the actor launch above, "
                                + ("one persistent launch" if sched == pr.PR_SCHED_FUSED else "one launch per step")}
    del mu
    return res


def main():
    if "--calibrate" in sys.argv[1:]:
        return calibrate()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--schedule", default="fused", choices=["stepwise", "fused"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-envs", type=int, default=192)
    ap.add_argument("--cpu-steps", type=int, default=1024)
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed side measurements (metrics, population, learner, replay): profiler runs "
                         "then see only the timed path's kernels")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also launch one plain elementwise copy of this many MiB (read + write that much each), "
                         "the known-size kernel hardware traffic counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (envs shard trivially across GPUs; no multi-GPU "
                 "path is built or measured). Use --gpus 1.")

    import torch
    from paper_2112_05923_amd import inputs, podrollout as pr

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = torch.device("cuda:0")
    w = inputs.WORKLOADS[args.workload]
    T, N, D, S = w.steps, w.n_envs, w.n_stocks, w.state_dim
    d = inputs.make_all_device(w, dev)
    sched = pr.PR_SCHED_FUSED if args.schedule == "fused" else pr.PR_SCHED_STEPWISE
    ro = pr.Rollout(pr.make_config(w, schedule=sched), d["price"], d["ind"], d["actor"], d["critic"])
    out = ro.alloc_buffers(T, value=True, logp=True, mu=False, shares=False)
    roll = dict(out)
    roll["value"] = None
    adv = torch.empty((T, N), dtype=torch.float32, device=dev)
    ret = torch.empty((T, N), dtype=torch.float32, device=dev)
    obs2d = out["obs"].view((T + 1) * N, S)
    val2d = out["value"].view((T + 1) * N, 1)

    def one_step(ev=None):
        ro.reset()
        if ev:
            ev[0].record()
        ro.step_T(T, d["noise"], roll)
        if ev:
            ev[1].record()
        ro.mlp_forward(pr.PR_NET_CRITIC, obs2d, val2d)
        if ev:
            ev[2].record()
        pr.compute_gae(out["reward"], out["value"], out["done"], w.gamma, w.lam, adv, ret)
        if ev:
            ev[3].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(events[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    if args.copy_calibration:
        src = torch.ones(args.copy_calibration << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one vectorised elementwise kernel: reads and writes copy_calibration MiB
        torch.cuda.synchronize()

    alone = {} if args.no_extras else stages_alone(torch, pr, inputs, w, d, ro, out, roll, obs2d, sched, dev)
    extras = {} if args.no_extras else side_measurements(torch, pr, inputs, w, d, out, roll, adv, ret, obs2d, val2d,
                                                         sched, dev)
    ms = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in events) / args.steps
    t_roll, t_critic, t_gae = ms(0, 1), ms(1, 2), ms(2, 3)
    env_steps = N * T
    value = env_steps * args.steps / dt

    flops_actor = inputs.mlp_flops_per_env_step(w, critic=False) * env_steps
    flops_critic = inputs.mlp_flops_per_env_step(w, critic=True) * (T + 1) * N
    env_bytes = inputs.bytes_per_env_step(w) * env_steps
    gae_bytes = 17 * env_steps
    mf = "mfma_bf16" if w.mlp_dtype else "mfma_fp32"
    stages = {
        "rollout_T": {"ms": t_roll, "actor_TFLOPs": flops_actor / t_roll / 1e9,
                      "env_algorithmic_GBps": env_bytes / t_roll / 1e6},
        "critic": {"ms": t_critic, "TFLOPs": flops_critic / t_critic / 1e9, "frac_mfma": flops_critic / t_critic / 1e9 / PEAK[mf][0]},
        "gae": {"ms": t_gae, "GBps": gae_bytes / t_gae / 1e6, "frac_hbm": gae_bytes / t_gae / 1e6 / PEAK["hbm"][0]},
    }
    # dominant kernel: the single launch that takes the largest share of a step
    if args.schedule == "fused":
        dom = {"kernel": "rollout_fused_kernel", "bound": "mfma", "achieved": flops_actor / t_roll / 1e9,
               "peak": PEAK[mf][0], "unit": "TFLOP/s", "ms_per_launch": t_roll}
    else:
        dom = {"kernel": "critic over the whole buffer (value_kernel / mlp_tiles_kernel / mlp_wide_kernel by shape)", "bound": "mfma", "achieved": flops_critic / t_critic / 1e9,
               "peak": PEAK[mf][0], "unit": "TFLOP/s", "ms_per_launch": t_critic}
    dom["frac"] = dom["achieved"] / dom["peak"]
    dom["traffic"] = recorded_traffic("fused" if args.schedule == "fused" else "critic", w.name)
    if not args.no_extras:
        mp = measured_peaks()
        dom["measured"] = mp
        if w.mlp_dtype:
            dom["frac_of_measured_mfma"] = dom["achieved"] / mp["mfma_bf16_TFLOPs"]
            stages["critic"]["frac_of_measured_mfma"] = stages["critic"]["TFLOPs"] / mp["mfma_bf16_TFLOPs"]
        stages["gae"]["frac_of_measured_read"] = stages["gae"]["GBps"] / mp["hbm_read_GBps"]

    res = {
        "metric": "env-steps/sec (transitions/s) on 1 MI355X; achieved HBM GB/s and MFMA %",
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.mlp_dtype else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={N} envs, D={D} stocks, K={w.n_ind} indicators, T={T} steps, "
                               f"MLP {S}-{w.hidden}-{w.hidden}-{{{D},1}}", "schedule": args.schedule,
                   "env_steps_per_step": env_steps},
        "roofline": dom,
        "stages": stages,
        "stages_alone": alone,
        "extras": extras,
    }
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        res["cpu_baseline"] = cpu_baseline(w, args.cpu_envs, min(args.cpu_steps, T), threads)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
