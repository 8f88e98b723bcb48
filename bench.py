#!/usr/bin/env python3
"""Benchmark of the fused rollout + GAE path on one MI355X.

One "step" = one msrl_rollout_gae call = T environment steps of every env
(observation, both networks, sampling, env move, reward, reset, trajectory
stores) followed by the GAE pass.  The default workload is the largest of the
five synthetic configurations (65536 envs x 10 agents, bf16 networks, T = 200).

Prints ONE JSON line: agent-steps/s of the whole call, the roofline of the
dominant kernel (the rollout kernel: MFMA-bound) from HIP-event timings taken
in this run, a second roofline object for the GAE kernel (HBM-bound), and the
CPU oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0


def mlp_flops_per_agent_step(cfg) -> int:
    """2 * MACs of the un-padded policy and value networks."""
    d, h, hh = cfg.obs_dim, cfg.hidden, (cfg.hidden_layers - 1) * cfg.hidden * cfg.hidden
    if getattr(cfg, "central_critic", False):  # the value network runs once per env, on N * d inputs
        return 2 * (d * h + hh + h * cfg.out_dim) + 2 * (cfg.value_in_dim * h + hh + h) // cfg.num_agents
    return 2 * ((d * h + hh + h * cfg.out_dim) + (d * h + hh + h))


def rollout_bytes_per_agent_step(cfg) -> int:
    act = 4 if cfg.dist == 0 else 4 * cfg.act_dim
    return 4 * cfg.obs_dim + act + 4 + 4 + 1 + 4  # obs, action, logp, reward, done, value


GAE_BYTES_PER_AGENT_STEP = 17  # r, V, d read; adv, ret written


def read_traffic(name: str):
    """HBM bytes per launch from the committed counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def read_mfma_issued(name: str, flops_per_mfma: float):
    """Flops of the MFMA instructions one launch issues (padding of inputs, outputs and rows included), from the
    committed counter summary (SQ_INSTS_MFMA per launch), if there is one."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^\|\s*SQ_INSTS_MFMA\s*\|\s*([0-9.eE+]+)\s*\|", open(path).read(), flags=re.M)
    return float(m.group(1)) * flops_per_mfma if m else None


def cpu_baseline(cfg, seed, seconds_target=15.0):
    """The oracle as it stands on the host cores, on the first envs of the same
    workload over the full T (envs are independent and keyed by global env id)."""
    from concurrent.futures import ThreadPoolExecutor
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import oracle_setup
    from oracle import ref

    env, pol, params, _ = oracle_setup(cfg, bias_std=0.0)

    def run(env0, n_env, T):
        st, g = ref.init(env, seed, env0, n_env)
        tr = ref.rollout(env, pol, seed, env0, st, g, params, T, want_logits=False)
        ref.gae(tr["rewards"], tr["values"], tr["dones"], cfg.gamma, cfg.lam)
        return n_env * cfg.num_agents * T

    # calibrate on one env for a few steps, then size the sample to the target time
    t0 = time.perf_counter()
    n = run(0, 1, 4)
    per_step = (time.perf_counter() - t0) / n
    n_env = int(max(1, min(cfg.num_envs, seconds_target / (per_step * cfg.num_agents * cfg.T))))
    t0 = time.perf_counter()
    n = run(0, n_env, cfg.T)
    dt1 = time.perf_counter() - t0
    one = n / dt1
    threads = min(16, os.cpu_count() or 1)
    per_thread = max(1, n_env // 2)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as pool:
        done = sum(pool.map(lambda k: run(k * per_thread, per_thread, cfg.T), range(threads)))
    dtn = time.perf_counter() - t0
    return {
        "value": one, "unit": "agent-steps/s", "cores": 1, "kind": "oracle",
        "sample": f"envs 0..{n_env - 1} of {cfg.num_envs}, all T={cfg.T} steps, rollout + GAE ({n} agent-steps, {dt1:.1f} s)",
        "all_cores": {"value": done / dtn, "cores": threads,
                      "sample": f"{threads} threads x {per_thread} envs ({done} agent-steps, {dtn:.1f} s)"},
    }


def other_config(B, synth, torch, idx, steps, with_cpu):
    """One of the smaller configurations in the same way as the headline one: the whole call, the rollout
    kernel alone (HIP events), its fraction of the MFMA peak of its dtype, and the oracle on a bounded sample."""
    cfg = synth.CONFIGS[idx]
    dyn = synth.make_dynamics(cfg) if cfg.kind == synth.LINGAUSS else (None, None)
    env_cfg, keep = B.make_env_cfg(cfg, *dyn)
    state = B.msrl_rollout_init(env_cfg, B.make_policy_cfg(cfg), cfg.env_seed)
    dparams = B.upload_params(cfg, synth.make_params(cfg))
    out = B.alloc_traj(cfg, cfg.T, logits=False, gae=True)
    T, steps_per_call = cfg.T, cfg.T * cfg.M
    for _ in range(2):
        B.msrl_rollout_gae(state, dparams, T, cfg.gamma, cfg.lam, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.msrl_rollout_gae(state, dparams, T, cfg.gamma, cfg.lam, out)
    torch.cuda.synchronize()
    ms_call = (time.perf_counter() - t0) / steps * 1e3
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    for k in range(steps):
        ev[k][0].record()
        B.msrl_rollout_step(state, dparams, T, out)
        ev[k][1].record()
    torch.cuda.synchronize()
    roll_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    shape = B.msrl_rollout_shape(state)
    B.msrl_rollout_destroy(state)
    dt_name = "bf16" if cfg.dtype == synth.BF16 else "f32"
    tf = mlp_flops_per_agent_step(cfg) * steps_per_call / (roll_ms * 1e-3) / 1e12
    res = {"workload": cfg.name, "dtype": dt_name, "rows_M": cfg.M, "T": T, "agent_steps_per_call": steps_per_call,
           "ms_per_call": ms_call, "agent_steps_per_s": steps_per_call / (ms_call * 1e-3),
           "rollout_ms_per_launch": roll_ms,
           "launch": {"workgroups": shape[0], "waves_per_workgroup": shape[1], "row_blocks_per_workgroup": shape[2]},
           "roofline": {"kernel": "rollout", "bound": "mfma", "achieved": tf, "peak": PEAK_TFLOPS[dt_name],
                        "unit": "TFLOP/s", "frac": tf / PEAK_TFLOPS[dt_name]},
           "hbm_GBps": (rollout_bytes_per_agent_step(cfg) + GAE_BYTES_PER_AGENT_STEP) * steps_per_call / (ms_call * 1e-3) / 1e9}
    if with_cpu:
        res["cpu_baseline"] = cpu_baseline(cfg, cfg.env_seed, seconds_target=3.0)
    del out
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="synthetic configuration 1..5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-phases", action="store_true", help="skip the env-only / MLP-only phase timings")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the figures of the smaller configurations")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this size (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_2210_00882_amd import binding as B, synth

    cfg = synth.CONFIGS[args.config]
    seed = cfg.env_seed
    params = synth.make_params(cfg)  # benchmark recipe: weights N(0, 1/fan_in), biases 0
    dyn = synth.make_dynamics(cfg) if cfg.kind == synth.LINGAUSS else (None, None)
    env_cfg, keep = B.make_env_cfg(cfg, *dyn)
    state = B.msrl_rollout_init(env_cfg, B.make_policy_cfg(cfg), seed)
    dparams = B.upload_params(cfg, params)
    launch_shape = B.msrl_rollout_shape(state)
    out = B.alloc_traj(cfg, cfg.T, logits=False, gae=True)
    T, M = cfg.T, cfg.M
    agent_steps = T * M

    def step():
        B.msrl_rollout_gae(state, dparams, T, cfg.gamma, cfg.lam, out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-kernel durations: the same two launches msrl_rollout_gae enqueues, issued
    # separately with HIP events between them on the stream they run on
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for k in range(args.steps):
        ev[k][0].record()
        B.msrl_rollout_step(state, dparams, T, out)
        ev[k][1].record()
        B.msrl_gae(out["rewards"], out["values"], out["dones"], cfg.gamma, cfg.lam, out["adv"], out["ret"])
        ev[k][2].record()
    torch.cuda.synchronize()
    roll_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    gae_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))

    dt_name = "bf16" if cfg.dtype == synth.BF16 else "f32"
    flops = mlp_flops_per_agent_step(cfg) * agent_steps
    achieved = flops / (roll_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "rollout", "bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[dt_name],
        "unit": "TFLOP/s", "frac": achieved / PEAK_TFLOPS[dt_name],
        "traffic": read_traffic(f"rollout_cfg{args.config}_pmc.md"),
        "ms_per_launch": roll_ms,
        "hbm_GBps": rollout_bytes_per_agent_step(cfg) * agent_steps / (roll_ms * 1e-3) / 1e9,
    }
    # the same on issued work: what the matrix pipe executes, padding included (32x32x16 bf16: 32768 flops per
    # instruction; 32x32x2 fp32: 4096)
    issued = read_mfma_issued(f"rollout_cfg{args.config}_units.md", 32768.0 if cfg.dtype == synth.BF16 else 4096.0)
    if issued:
        roofline["mfma_issued"] = {"flops_per_launch": issued, "over_algorithmic": issued / flops,
                                   "frac": issued / (roll_ms * 1e-3) / 1e12 / PEAK_TFLOPS[dt_name]}
    gae_achieved = GAE_BYTES_PER_AGENT_STEP * agent_steps / (gae_ms * 1e-3) / 1e9
    roofline_gae = {
        "kernel": "gae", "bound": "hbm", "achieved": gae_achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": gae_achieved / PEAK_HBM_GBS, "traffic": read_traffic(f"gae_cfg{args.config}_pmc.md"),
        "ms_per_launch": gae_ms,
    }

    # phase rooflines: the same kernel with the networks skipped (env phase, HBM-bound: every
    # trajectory store is kept) and with only the networks (MLP phase, MFMA-bound)
    phases = None
    if not args.no_phases:
        phases = {}
        for name, phase in (("env", B.MSRL_PHASE_ENV), ("mlp", B.MSRL_PHASE_MLP)):
            try:
                B.msrl_measure_phase(state, dparams, T, out, phase)
            except B.MsrlError:
                continue  # variant not compiled for this configuration
            e0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
            e1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
            for k in range(args.steps):
                e0[k].record()
                B.msrl_measure_phase(state, dparams, T, out, phase)
                e1[k].record()
            torch.cuda.synchronize()
            ms = float(np.mean([a.elapsed_time(b) for a, b in zip(e0, e1)]))
            if name == "env":
                gbs = rollout_bytes_per_agent_step(cfg) * agent_steps / (ms * 1e-3) / 1e9
                phases[name] = {"bound": "hbm", "ms_per_launch": ms, "achieved": gbs, "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
            else:
                tf = flops / (ms * 1e-3) / 1e12
                phases[name] = {"bound": "mfma", "ms_per_launch": ms, "achieved": tf, "peak": PEAK_TFLOPS[dt_name],
                                "unit": "TFLOP/s", "frac": tf / PEAK_TFLOPS[dt_name]}

        # the step-granular calls (actor fragment, environment fragment) at the same batch size
        try:
            obs1 = torch.empty((M, cfg.obs_dim), dtype=torch.float32, device="cuda")
            B.msrl_observe(state, obs1)
            a1, lp1, v1 = out["actions"][0], out["logp"][0], out["values"][0]
            r1, d1 = out["rewards"][0], out["dones"][0]
            # (short calls: enough untimed ones first that the timed ones run at the clock of a busy device)
            reps, warm = 30, 30
            for name in ("act", "env_step"):
                ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for k in range(reps + warm):
                    if k == warm:
                        ev0.record()
                    if name == "act":   # (parameters passed once; later calls reuse their re-ordered image)
                        B.msrl_act(state, dparams if k == 0 else None, obs1, a1, lp1, v1)
                    else:
                        B.msrl_env_step(state, a1, r1, d1, obs1)
                ev1.record()
                torch.cuda.synchronize()
                ms = ev0.elapsed_time(ev1) / reps
                if name == "act":
                    tf = mlp_flops_per_agent_step(cfg) * M / (ms * 1e-3) / 1e12
                    phases[name] = {"bound": "mfma", "ms_per_call": ms, "achieved": tf, "peak": PEAK_TFLOPS[dt_name],
                                    "unit": "TFLOP/s", "frac": tf / PEAK_TFLOPS[dt_name], "rows": M}
                else:
                    act_b = 4 if cfg.dist == 0 else 4 * cfg.act_dim
                    state_b = 8 * (cfg.env_state_size + 2) / cfg.num_agents   # state + counter, read and written
                    gbs = (4 * cfg.obs_dim + act_b + 5 + state_b) * M / (ms * 1e-3) / 1e9
                    phases[name] = {"bound": "hbm", "ms_per_call": ms, "achieved": gbs, "peak": PEAK_HBM_GBS,
                                    "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "rows": M}
        except B.MsrlError:
            pass

        # the learner's minibatch gradient (next row of the path) on rows of the trajectory just produced
        try:
            rows = int(min(T * M, 512 * 1024))
            learner = B.msrl_learner_init(B.make_policy_cfg(cfg), rows)
            master = torch.from_numpy(np.ascontiguousarray(params, dtype=np.float32)).cuda()
            grad = torch.empty_like(master)
            flat = lambda t: t.reshape(-1, *t.shape[2:])[:rows]
            batch = (flat(out["obs"][:T]), flat(out["actions"]), flat(out["logp"]), flat(out["adv"]), flat(out["ret"]))
            pc = B.make_ppo_cfg()
            reps, warm = 10, 5
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for k in range(reps + warm):
                if k == warm:
                    ev0.record()
                B.msrl_ppo_grad(learner, master, *batch, pc, grad)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / reps
            B.msrl_learner_destroy(learner)
            # forward + backward through the activations + weight gradients; no gradient w.r.t. the observation
            fl = (3 * mlp_flops_per_agent_step(cfg) - 2 * 2 * cfg.obs_dim * cfg.hidden) * rows
            tf = fl / (ms * 1e-3) / 1e12
            phases["learner_grad"] = {"bound": "mfma", "ms_per_call": ms, "rows": rows, "achieved": tf,
                                      "peak": PEAK_TFLOPS[dt_name], "unit": "TFLOP/s", "frac": tf / PEAK_TFLOPS[dt_name],
                                      "rows_per_s": rows / (ms * 1e-3)}
            if cfg.dtype == synth.BF16 and cfg.hidden > 64 and cfg.dist == synth.CATEGORICAL:
                # What the on-chip path moves through HBM per row by design (bf16 tiles, both networks): x once,
                # h1, h2, dz2, dz1, dy per network, each written by the row kernel and read by the weight
                # gradients, h2 read once more by the row kernel; the observation row and the loss inputs per network.
                H, D = cfg.hidden, cfg.obs_dim
                kt1 = 2 if D + 2 <= 32 else 4
                tiles_b = 2 * (4 * H * 2 + 32) + 16 * kt1 * 2
                per_row = 2 * tiles_b + 2 * H * 2 + 2 * (4 * D + 12)
                gbs = per_row * rows / (ms * 1e-3) / 1e9
                phases["learner_grad"]["hbm"] = {"bytes_per_call": per_row * rows, "achieved": gbs, "peak": PEAK_HBM_GBS,
                                                 "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
            del master, grad
        except B.MsrlError:
            pass

        # the same rollout with the network depth of the paper's evaluation (seven layers = six hidden
        # layers and the output layer), if a kernel for it is compiled
        try:
            deep = cfg.with_(hidden_layers=6)
            dstate = B.msrl_rollout_init(env_cfg, B.make_policy_cfg(deep), seed)
            dp = B.upload_params(deep, synth.make_params(deep))
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for k in range(3):
                if k == 1:
                    ev0.record()
                B.msrl_rollout_step(dstate, dp, T, out)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / 2
            B.msrl_rollout_destroy(dstate)
            tf = mlp_flops_per_agent_step(deep) * agent_steps / (ms * 1e-3) / 1e12
            phases["rollout_6_hidden_layers"] = {"bound": "mfma", "ms_per_launch": ms, "achieved": tf,
                                                 "peak": PEAK_TFLOPS[dt_name], "unit": "TFLOP/s",
                                                 "frac": tf / PEAK_TFLOPS[dt_name],
                                                 "agent_steps_per_s": agent_steps / (ms * 1e-3)}
            del dp
        except B.MsrlError:
            pass

        # the same rollout with a centralised critic (multi-agent PPO, section 2.1 of the paper): the value
        # network takes the joint observation of an env and runs once per env
        try:
            cen = cfg.with_(central_critic=True)
            cstate = B.msrl_rollout_init(env_cfg, B.make_policy_cfg(cen), seed)
            cp = B.upload_params(cen, synth.make_params(cen))
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for k in range(4):
                if k == 1:
                    ev0.record()
                B.msrl_rollout_step(cstate, cp, T, out)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / 3
            B.msrl_rollout_destroy(cstate)
            tf = mlp_flops_per_agent_step(cen) * agent_steps / (ms * 1e-3) / 1e12
            phases["rollout_central_critic"] = {"bound": "mfma", "ms_per_launch": ms, "achieved": tf,
                                                "peak": PEAK_TFLOPS[dt_name], "unit": "TFLOP/s",
                                                "frac": tf / PEAK_TFLOPS[dt_name],
                                                "agent_steps_per_s": agent_steps / (ms * 1e-3)}
            del cp
        except B.MsrlError:
            pass

        # the same gradient with a centralised critic (value network on the joint observation of an env's
        # agents: a tenth of the rows, ten times the input width), on the same rows
        try:
            cen = cfg.with_(central_critic=True)
            rows = int(min(T * M, 512 * 1024)) // cen.num_agents * cen.num_agents
            learner = B.msrl_learner_init(B.make_policy_cfg(cen), rows)
            master = torch.from_numpy(np.ascontiguousarray(synth.make_params(cen), dtype=np.float32)).cuda()
            grad = torch.empty_like(master)
            flat = lambda t: t.reshape(-1, *t.shape[2:])[:rows]
            batch = (flat(out["obs"][:T]), flat(out["actions"]), flat(out["logp"]), flat(out["adv"]), flat(out["ret"]))
            pc = B.make_ppo_cfg()
            reps, warm = 10, 5
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for k in range(reps + warm):
                if k == warm:
                    ev0.record()
                B.msrl_ppo_grad(learner, master, *batch, pc, grad)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / reps
            B.msrl_learner_destroy(learner)
            fl = (3 * mlp_flops_per_agent_step(cen) - 2 * cen.obs_dim * cen.hidden
                  - 2 * cen.value_in_dim * cen.hidden // cen.num_agents) * rows
            tf = fl / (ms * 1e-3) / 1e12
            phases["learner_grad_central_critic"] = {"bound": "mfma", "ms_per_call": ms, "rows": rows, "achieved": tf,
                                                     "peak": PEAK_TFLOPS[dt_name], "unit": "TFLOP/s",
                                                     "frac": tf / PEAK_TFLOPS[dt_name], "rows_per_s": rows / (ms * 1e-3)}
            del master, grad
        except B.MsrlError:
            pass

        # the pursuit ("tag") env at the scale of the paper's GPU-only experiment (Fig. 10: up to
        # 100,000 agents on one GPU): 25,000 envs x (3 chasers + 1 runner), 64-unit bf16 networks per role
        try:
            tcfg = synth.tag("tag_100k_agents", 25000, 3, 1, 2, 64, 100, 25)
            tenv, tkeep = B.make_env_cfg(tcfg, None, None)
            tstate = B.msrl_rollout_init(tenv, B.make_policy_cfg(tcfg), seed)
            tparams = B.upload_params(tcfg, synth.make_params(tcfg))
            tout = B.alloc_traj(tcfg, tcfg.T, logits=False, gae=True)
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps, warm = 10, 5
            for k in range(reps + warm):
                if k == warm:
                    ev0.record()
                B.msrl_rollout_gae(tstate, tparams, tcfg.T, tcfg.gamma, tcfg.lam, tout)
            ev1.record()
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1) / reps
            B.msrl_rollout_destroy(tstate)
            steps_t = tcfg.T * tcfg.M
            gbs = (rollout_bytes_per_agent_step(tcfg) + GAE_BYTES_PER_AGENT_STEP) * steps_t / (ms * 1e-3) / 1e9
            tf = mlp_flops_per_agent_step(tcfg) * steps_t / (ms * 1e-3) / 1e12
            phases["tag_100k_agents"] = {"bound": "hbm", "ms_per_call": ms, "achieved": gbs, "peak": PEAK_HBM_GBS,
                                         "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "T": tcfg.T,
                                         "agent_steps_per_s": steps_t / (ms * 1e-3), "mfma_TFLOPs": tf}
            del tout, tparams
        except B.MsrlError:
            pass

        # one training iteration of Listing 1 at that scale: a 25-step episode of 100,000 agents (rollout + GAE),
        # then the learner's update of both roles on the 2.5 M rows it produced (one pass, four minibatches per
        # role; a role's rows are named by an msrl_row_select, nothing is copied) -- the kind of figure the paper's
        # "time per episode" (Fig. 10b) is, on a different task definition
        try:
            ecfg = synth.tag("tag_100k_agents_episode", 25000, 3, 1, 2, 64, 25, 25)
            eenv, ekeep = B.make_env_cfg(ecfg, None, None)
            estate = B.msrl_rollout_init(eenv, B.make_policy_cfg(ecfg), seed)
            one_role = B.make_policy_cfg(ecfg)
            one_role.roles = 1
            n_role = B.msrl_param_count(one_role)
            master = torch.from_numpy(synth.make_params(ecfg).astype(np.float32)).cuda()
            m1, v1 = torch.zeros_like(master), torch.zeros_like(master)
            acting = torch.empty(master.numel(), dtype=torch.bfloat16, device="cuda")
            eout = B.alloc_traj(ecfg, ecfg.T, logits=False, gae=True)
            N_, NC_ = ecfg.num_agents, ecfg.num_chasers
            sets = [B.msrl_row_select(N_, 0, NC_), B.msrl_row_select(N_, NC_, N_ - NC_)]   # the rows of each role
            counts = [ecfg.T * ecfg.num_envs * r.count for r in sets]
            mbs = 4
            learners = [B.msrl_learner_init(one_role, -(-c // mbs) + mbs) for c in counts]
            pc = B.make_ppo_cfg(lr=3e-4)
            flat = lambda t: t.reshape(-1, *t.shape[2:])
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            reps, warm, t_roll, ms_it, ksteps = 6, 3, 0.0, 0.0, [0, 0]
            for k in range(reps + warm):
                evs[0].record()
                B.msrl_params_cast(master, acting, B.MSRL_BF16)
                B.msrl_rollout_gae(estate, acting, ecfg.T, ecfg.gamma, ecfg.lam, eout)
                evs[1].record()
                batch = [flat(eout["obs"][:ecfg.T]), flat(eout["actions"]), flat(eout["logp"]), flat(eout["adv"]),
                         flat(eout["ret"])]
                for r in range(2):
                    sl = slice(r * n_role, (r + 1) * n_role)
                    ksteps[r] = B.msrl_ppo_update(learners[r], master[sl], m1[sl], v1[sl], ksteps[r], 1, mbs, *batch, pc,
                                                  rows=sets[r])
                evs[2].record()
                torch.cuda.synchronize()
                if k >= warm:
                    t_roll += evs[0].elapsed_time(evs[1])
                    ms_it += evs[0].elapsed_time(evs[2])
            for Lr in learners:
                B.msrl_learner_destroy(Lr)
            B.msrl_rollout_destroy(estate)
            phases["tag_100k_agents_train_iteration"] = {
                "ms_per_iteration": ms_it / reps, "rollout_gae_ms": t_roll / reps, "update_ms": (ms_it - t_roll) / reps,
                "rows": ecfg.T * ecfg.M, "episode_steps": ecfg.T, "update": "1 pass, 4 minibatches per role",
                "agent_steps_per_s": ecfg.T * ecfg.M / (ms_it / reps * 1e-3)}
            del eout, master, m1, v1, acting
        except B.MsrlError:
            pass

        # in-kernel clocks of the fused kernel: where one step of one workgroup spends its cycles
        stamps = torch.zeros(1024, dtype=torch.float32, device="cuda")
        try:
            B.msrl_measure_phase(state, dparams, T, dict(out, logits=stamps), B.MSRL_PHASE_CLOCKS)
            torch.cuda.synchronize()
            c = stamps[:256].cpu().numpy().reshape(8, 32)
            names = {1: "obs_build_store", 2: "policy_layer1", 3: "policy_stage0", 4: "policy_stage1",
                     5: "policy_stage2", 6: "policy_stage3", 8: "value_layer1", 9: "value_stage0",
                     10: "value_stage1", 11: "value_stage2", 12: "value_stage3", 14: "outputs",
                     15: "sample_move", 16: "reward_done_reset"}
            order = sorted(names)
            mean = c.mean(0)
            prev, split = 0.0, {}
            for i in order:
                split[names[i]] = float(mean[i] - prev)
                prev = float(mean[i])
            phases["clocks"] = {"unit": "shader-clock cycles, mean over the 8 waves of workgroup 0, step T/2",
                                "step_total": prev, "split": split,
                                # of which: in the waits at the ten stage barriers of the step (copies landed + barrier)
                                "stage_barrier_waits": float(mean[20]),
                                "stage_barrier_waits_per_wave": [float(x) for x in c[:, 20]]}
        except B.MsrlError:
            pass  # variant not compiled for this configuration

    if args.copy_calibration:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # reads and writes copy_calibration MiB each
        torch.cuda.synchronize()
        del src, dst

    B.msrl_rollout_destroy(state)
    del out
    torch.cuda.empty_cache()

    # the smaller configurations (the parity-test cases) in the same JSON line, for the record
    others = None
    if not args.no_other_configs:
        others = {}
        for idx in sorted(synth.CONFIGS):
            if idx != args.config:
                others[f"cfg{idx}"] = other_config(B, synth, torch, idx, max(3, args.steps), not args.no_cpu_baseline)
        torch.cuda.empty_cache()

    result = {
        "metric": "agent-steps/sec of fused rollout+GAE at 1 GPU",
        "value": agent_steps / (ms_per_step * 1e-3),
        "unit": "agent-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt_name, "data": "synthetic",
        "config": {"workload": cfg.name, "num_envs": cfg.num_envs, "num_agents": cfg.num_agents,
                   "rows_M": M, "T": T, "obs_dim": cfg.obs_dim, "hidden": cfg.hidden,
                   "agent_steps_per_step": agent_steps,
                   "launch": {"workgroups": launch_shape[0], "waves_per_workgroup": launch_shape[1],
                              "row_blocks_per_workgroup": launch_shape[2]}},
        "roofline": roofline,
        "roofline_gae": roofline_gae,
        "phases": phases,
        "other_configs": others,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(cfg, seed),
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
