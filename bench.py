#!/usr/bin/env python3
"""Benchmark of the fused MPE simple-spread rollout on one MI355X.

A "step" here is one pass of the whole hot path over one batch: one mpe_rollout call of
T = 128 fused steps (policy MLP on MFMA -> Gumbel-max -> transition -> reward/auto-reset ->
observation -> trajectory stores) at 65,536 environments x 3 agents, inputs resident in HBM.
The same shape is also timed env-only (seeded uniform actions) for the HBM-roofline figure,
and the CPU oracle is timed on a bounded sample of the same workload as a baseline.

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix; the fp32 vector peak is the same number
KERNEL_SOURCES = ("paper_2311_10090_amd/csrc", "include")


def _code_only(text):
    """C++ source without its comments and with every run of white space collapsed to one blank (string and
    character literals are kept as they are)."""
    out, i, n = [], 0, len(text)
    while i < n:
        c = text[i]
        if c in "\"'":
            j = i + 1
            while j < n and text[j] != c:
                j += 2 if text[j] == "\\" else 1
            out.append(text[i:j + 1])
            i = j + 1
        elif text.startswith("//", i):
            j = text.find("\n", i)
            i = n if j < 0 else j
        elif text.startswith("/*", i):
            j = text.find("*/", i + 2)
            i = n if j < 0 else j + 2
            out.append(" ")
        else:
            out.append(c)
            i += 1
    return " ".join("".join(out).split())


def kernel_source_hash():
    """sha256 over the code of the HIP sources and the header (comments and white space left out): counter
    figures stored under profiles/ carry the hash of the sources they were measured on, and are reported only
    while it still matches."""
    import hashlib
    h = hashlib.sha256()
    for d in KERNEL_SOURCES:
        for name in sorted(os.listdir(os.path.join(ROOT, d))):
            if name.endswith((".hip", ".h")):
                h.update(name.encode())
                h.update(_code_only(open(os.path.join(ROOT, d, name), encoding="utf-8").read()).encode())
    return h.hexdigest()


def spread_env(synth, *a, **kw):
    from paper_2311_10090_amd.binding import MpeConfig, MpeEnv
    return MpeEnv(MpeConfig(**synth.spread_config(*a, **kw)))


def tag_env(synth, *a, **kw):
    from paper_2311_10090_amd.binding import MpeConfig, MpeEnv
    return MpeEnv(MpeConfig(**synth.tag_config(*a, **kw)))


def to_dev(arrs):
    import numpy as np
    import torch
    return [torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0") for a in arrs]


def flops_per_agent_step(D, H, A=5):
    return 2 * (D * H + H * H + H * A)          # 11,136 for 18 -> 64 -> 64 -> 5


def bytes_per_env_step(N, D):
    return N * D * 4 + N + 4 + 1                  # obs + actions + reward + done: 224 for N = 3


def time_rollouts(env, T, bufs, steps, warmup):
    import torch
    for _ in range(warmup):
        env.rollout(T, *bufs)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in evs:
        a.record()                 # on torch's current stream: the stream the kernel is launched on
        env.rollout(T, *bufs)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in evs]
    return wall, kern_ms


def cpu_baseline(workload, weights, T, seed, target_seconds=12.0):
    """Time the oracle on envs 0..n-1 of the same workload.  n is sized from a short probe so that
    the timed run takes about target_seconds on this machine's cores (bounded by the workload)."""
    from oracle import Oracle, OracleConfig
    from paper_2311_10090_amd import synth
    cores = max(1, min(os.cpu_count() or 1, 16))

    def run(n, threads=cores):
        orc = Oracle(OracleConfig(**synth.spread_config(n, workload.num_agents, 1, workload.hidden, workload.weight_dtype,
                                                        as_f32=True)), threads=threads)
        orc.set_policy(*weights)
        orc.reset(seed)
        t0 = time.perf_counter()
        orc.rollout(T, want_obs=False)
        return time.perf_counter() - t0

    probe_n = min(1024, workload.num_envs)
    probe = run(probe_n)
    n = int(min(workload.num_envs, max(probe_n, probe_n * target_seconds / max(probe, 1e-3))))
    n -= n % 64 if n >= 64 else 0
    dt = run(n)
    n1 = max(64, n // (4 * cores))          # single-thread figure on a sample sized for ~1/4 of the time
    dt1 = run(n1, threads=1)
    return {"value": n * workload.num_agents * T / dt, "unit": "agent-steps/s", "cores": cores,
            "kind": "oracle", "seconds": round(dt, 3),
            "one_thread": {"value": n1 * workload.num_agents * T / dt1, "envs": n1, "seconds": round(dt1, 3)},
            "sample": "envs 0..%d of the same workload (same seed, same weights), %d fused steps, "
                      "fp64 scalar C++ oracle, %d threads over contiguous env ranges" % (n - 1, T, cores)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target duration of the oracle timing")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of the observation trajectory (for counter calibration)")
    ap.add_argument("--only-headline", action="store_true", help="skip the secondary workloads (short profiler runs)")
    ap.add_argument("--print-source-hash", action="store_true")
    args = ap.parse_args()
    if args.print_source_hash:
        print(kernel_source_hash())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (independent envs shard trivially, but no "
              "multi-GPU path is built); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2311_10090_amd import synth

    assert torch.cuda.is_available(), "bench.py needs an MI355X; there is no CPU fallback"
    wl = synth.WORKLOADS[args.workload]
    N, D, H, T, seed = wl.num_agents, wl.obs_dim, wl.hidden, wl.T, 1
    TE = wl.total_envs

    # ---- fused rollout (the metric)
    env = spread_env(synth, wl.num_envs, N, wl.num_runs, H, wl.weight_dtype)
    weights = synth.policy_weights(0, wl.num_runs, D, H)
    env.set_policy(*to_dev(weights))
    env.reset(seed)
    bufs = env.empty_traj(T)
    # One plain copy of known size (the observation trajectory onto a second buffer), outside every timed
    # region: under `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` this dispatch calibrates the byte counters.
    if args.calibration_copy:
        spare = torch.empty_like(bufs[0])
        spare.copy_(bufs[0])
        torch.cuda.synchronize()
        del spare
    wall, kern_ms = time_rollouts(env, T, bufs, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    agent_steps = TE * N * T
    value = agent_steps / (wall / args.steps)
    kavg = float(np.mean(kern_ms))
    tflops = flops_per_agent_step(D, H) * agent_steps / (kavg * 1e-3) / 1e12
    fused_gbs = bytes_per_env_step(N, D) * TE * T / (kavg * 1e-3) / 1e9
    # other seeds (different initial states, hence different contact patterns), a few calls each
    by_seed = {str(seed): value}
    for other in (2, 3):
        env.reset(other)
        w_o, _ = time_rollouts(env, T, bufs, max(3, args.steps // 3), 1)
        by_seed[str(other)] = agent_steps / (w_o / max(3, args.steps // 3))
    # a little sanity: trajectories were really produced
    done_sum = int(bufs[3].sum().item())
    assert done_sum == TE * (T // synth.MAX_EPISODE_STEPS) or done_sum == TE * (T // synth.MAX_EPISODE_STEPS + 1)
    env.close()

    # ---- env-only rollout, same shape (HBM roofline figure)
    env2 = spread_env(synth, wl.num_envs, N, wl.num_runs, 0, 0)
    env2.reset(seed)
    wall2, kern2 = time_rollouts(env2, T, bufs, args.steps, args.warmup)
    k2avg = float(np.mean(kern2))
    env_gbs = bytes_per_env_step(N, D) * TE * T / (k2avg * 1e-3) / 1e9
    # single mpe_step calls (launch-latency dominated at this size; reported, not a roofline figure)
    actions = torch.zeros((TE, N), dtype=torch.uint8, device="cuda")
    sbufs = (env2.empty_obs(), torch.empty(TE, dtype=torch.float32, device="cuda"),
             torch.empty(TE, dtype=torch.uint8, device="cuda"))
    for _ in range(5):
        env2.step(actions, *sbufs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_single = 200
    for _ in range(n_single):
        env2.step(actions, *sbufs)
    torch.cuda.synchronize()
    step_us = (time.perf_counter() - t0) / n_single * 1e6
    env2.close()

    # the mixed per-agent reward mode on the same shape (rewards [T][TE][N]; a few calls)
    mixed = {}
    extras = not args.only_headline
    if extras and (wl.weight_dtype == 0 or N == 10):
        k = max(3, args.steps // 3)
        env3 = spread_env(synth, wl.num_envs, N, wl.num_runs, H, wl.weight_dtype, reward_mode=1, local_ratio=0.5)
        env3.set_policy(*to_dev(weights))
        env3.reset(seed)
        b3 = env3.empty_traj(T)
        w3, k3 = time_rollouts(env3, T, b3, k, 2)
        env3.set_policy()
        env3.reset(seed)
        w4, k4 = time_rollouts(env3, T, b3, k, 2)
        mixed = {"fused_agent_steps_per_s": agent_steps / (w3 / k), "fused_kernel_ms_avg": float(np.mean(k3)),
                 "env_only_agent_steps_per_s": agent_steps / (w4 / k), "env_only_kernel_ms_avg": float(np.mean(k4)),
                 "bytes_per_env_step": bytes_per_env_step(N, D) + 4 * (N - 1),
                 "note": "MPE_REWARD_MIXED, local_ratio 0.5; env-only at N <= 3 uses the general one-wave-per-64-envs kernel"}
        env3.close()
        del b3

    # actor-critic rollout on the same shape (adds log-prob, value and bootstrap value outputs)
    ac = {}
    if extras and wl.weight_dtype == 0 and wl.num_runs == 1:
        k = max(3, args.steps // 3)
        env4 = spread_env(synth, wl.num_envs, N, wl.num_runs, H, 0)
        env4.set_policy(*to_dev(weights))
        env4.set_critic(*to_dev(synth.critic_weights(0, wl.num_runs, D, H)))
        env4.reset(seed)
        b4 = env4.empty_traj_ac(T)
        for _ in range(2):
            env4.rollout_ac(T, *b4)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            env4.rollout_ac(T, *b4)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / k
        ac = {"agent_steps_per_s": agent_steps / dt, "ms_per_rollout": dt * 1e3,
              "flop_per_agent_step": flops_per_agent_step(D, H) + flops_per_agent_step(D, H, 1),
              "fp32_equivalent_TFLOPs": (flops_per_agent_step(D, H) + flops_per_agent_step(D, H, 1)) * agent_steps / dt / 1e12,
              "bytes_per_env_step": bytes_per_env_step(N, D) + 8 * N,
              "note": "mpe_rollout_ac: policy + critic (6N->64->64->1); 256-env blocks of four sync groups when they fill half the chip, else 64-env blocks"}
        env4.close()
        del b4

    # the same shape with bf16 weights and layer inputs (fp32 accumulate), as defined by the oracle's bf16 mode
    bf = {}
    if extras and wl.weight_dtype == 0:
        k = max(3, args.steps // 3)
        env5 = spread_env(synth, wl.num_envs, N, wl.num_runs, H, 1)
        env5.set_policy(*to_dev(weights))
        env5.reset(seed)
        b5 = env5.empty_traj(T)
        w5, k5 = time_rollouts(env5, T, b5, k, 2)
        bf = {"agent_steps_per_s": agent_steps / (w5 / k), "kernel_ms_avg": float(np.mean(k5)),
              "hbm_GBs": bytes_per_env_step(N, D) * TE * T / (float(np.mean(k5)) * 1e-3) / 1e9,
              "note": "weight_dtype = MPE_WEIGHTS_BF16: one bf16 matrix instruction per product, no operand split"}
        env5.close()
        del b5

    # the paper's own many-seeds setting: 1,024 training runs (App. F) of 16 parallel envs each (App. G, IPPO
    # on MPE), every run with its own policy weights, and the whole batch at several sizes
    runs16 = {}
    if extras and args.workload == "cfg2":
        k = max(3, args.steps // 3)
        for nruns, per_run in ((1024, 16), (1024, 32)):
            env7 = spread_env(synth, per_run, N, nruns, H, 0)
            env7.set_policy(*to_dev(synth.policy_weights(0, nruns, D, H)))
            env7.reset(seed)
            b7 = env7.empty_traj(T)
            w7, k7 = time_rollouts(env7, T, b7, k, 2)
            runs16["%d_runs_x_%d_envs" % (nruns, per_run)] = {
                "agent_steps_per_s": nruns * per_run * N * T / (w7 / k), "kernel_ms_avg": float(np.mean(k7))}
            env7.close()
            del b7
        runs16["note"] = ("one set of weights per run; runs of 16 envs x 3 agents are blocks of 48 rows + 16 padding rows "
                          "in two wavefronts; multiples of 64 envs per run (cfg4) are the fast shape")

    # second scenario (predator-prey, 3 adversaries + 1 good agent + 2 obstacles) at the same number of
    # envs and steps: fused fp32 policy 16 -> 64 -> 64 -> 5 and env-only with uniform actions
    tag = {}
    if extras and args.workload == "cfg2":
        k = max(3, args.steps // 3)
        tN, tL, tA = 4, 2, 3
        tD = synth.tag_obs_dim(tN, tL, tA)
        t_bytes = tN * tD * 4 + tN + 4 * tN + 1                 # obs + actions + per-agent rewards + done: 277
        t_steps = wl.num_envs * tN * T
        for name, hidden, wd6 in (("fused", H, 0), ("fused_bf16", H, 1), ("env_only", 0, 0)):
            env6 = tag_env(synth, wl.num_envs, tN, tL, tA, 1, hidden, wd6)
            if hidden:
                env6.set_policy(*to_dev(synth.policy_weights(0, 1, tD, hidden)))
            env6.reset(seed)
            b6 = env6.empty_traj(T)
            w6, k6 = time_rollouts(env6, T, b6, k, 2)
            ms6 = float(np.mean(k6))
            tag[name] = {"agent_steps_per_s": t_steps / (w6 / k), "kernel_ms_avg": ms6,
                         "hbm_GBs": t_bytes * wl.num_envs * T / (ms6 * 1e-3) / 1e9,
                         "hbm_frac": t_bytes * wl.num_envs * T / (ms6 * 1e-3) / 1e9 / HBM_PEAK_GBS}
            if hidden and wd6 == 0:
                tf = flops_per_agent_step(tD, hidden) * t_steps / (ms6 * 1e-3) / 1e12
                tag[name].update({"flop_per_agent_step": flops_per_agent_step(tD, hidden), "fp32_equivalent_TFLOPs": tf,
                                  "frac_of_fp32_matrix_peak": tf / MFMA_FP32_PEAK_TFLOPS})
            env6.close()
            del b6
        # actor-critic rollout of the same scenario (policy + critic of the same shape with one output)
        env6 = tag_env(synth, wl.num_envs, tN, tL, tA, 1, H)
        env6.set_policy(*to_dev(synth.policy_weights(0, 1, tD, H)))
        env6.set_critic(*to_dev(synth.critic_weights(0, 1, tD, H)))
        env6.reset(seed)
        b6 = env6.empty_traj_ac(T)
        for _ in range(2):
            env6.rollout_ac(T, *b6)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            env6.rollout_ac(T, *b6)
        torch.cuda.synchronize()
        dt6 = (time.perf_counter() - t0) / k
        ac_flop = flops_per_agent_step(tD, H) + flops_per_agent_step(tD, H, 1)
        tag["actor_critic"] = {"agent_steps_per_s": t_steps / dt6, "ms_per_rollout": dt6 * 1e3,
                               "flop_per_agent_step": ac_flop, "fp32_equivalent_TFLOPs": ac_flop * t_steps / dt6 / 1e12,
                               "frac_of_fp32_matrix_peak": ac_flop * t_steps / dt6 / 1e12 / MFMA_FP32_PEAK_TFLOPS,
                               "note": "mpe_rollout_ac, wall time per call; 128-env blocks of 8 wavefronts around both staged networks"}
        env6.close()
        del b6
        tag["config"] = {"scenario": "MPE_SCENARIO_TAG", "envs": wl.num_envs, "agents": tN, "adversaries": tA,
                         "landmarks": tL, "obs_dim": tD, "T": T, "bytes_per_env_step": t_bytes,
                         "kernel": "tag_rollout_kernel (lane per agent; policy / uniform variants)"}

    # recurrent policy (GRU 128, bf16) on the headline env shape
    gru = {}
    if extras and args.workload == "cfg2":
        k = max(3, args.steps // 3)
        env7 = spread_env(synth, wl.num_envs, N, 1, 128, 1)
        env7.set_gru_policy(*to_dev(synth.gru_weights(0, 1, D)))
        env7.reset(seed)
        b7 = env7.empty_traj(T)
        w7, k7 = time_rollouts(env7, T, b7, k, 2)
        ms7 = float(np.mean(k7))
        g_flop = 2 * (D * 128 + 2 * 128 * 384 + 128 * 128 + 128 * 5)       # 235,264 per agent-step
        g_tf = g_flop * agent_steps / (ms7 * 1e-3) / 1e12
        gru = {"agent_steps_per_s": agent_steps / (w7 / k), "kernel_ms_avg": ms7, "flop_per_agent_step": g_flop,
               "roofline": {"bound": "mfma", "achieved": g_tf, "peak": 2500.0, "unit": "TFLOP/s", "frac": g_tf / 2500.0},
               "dtype": "bf16xbf16->f32", "kernel": "rollout_gru_kernel<3> (weight-stationary, 8 wavefronts per 64 envs)",
               "note": "mpe_set_gru_policy: 18 -> 128 tanh -> GRU 128 -> 128 tanh -> 5; carried state fp32"}
        # the recurrent actor-critic on the same shape: critic head on the new carried state, bootstrap pass
        env7.set_gru_critic(*to_dev(synth.gru_critic_weights(0, 1)))
        env7.reset(seed)
        b7 = env7.empty_traj_ac(T)
        for _ in range(2):
            env7.rollout_ac(T, *b7)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            env7.rollout_ac(T, *b7)
        torch.cuda.synchronize()
        dt7 = (time.perf_counter() - t0) / k
        gc_flop = g_flop + 2 * (128 * 128 + 128)
        gru["actor_critic"] = {"agent_steps_per_s": agent_steps / dt7, "ms_per_rollout": dt7 * 1e3,
                               "flop_per_agent_step": gc_flop, "TFLOPs": gc_flop * agent_steps / dt7 / 1e12,
                               "note": "mpe_set_gru_critic + mpe_rollout_ac, wall time per call; block shapes of the plain recurrent rollout"}
        env7.close()
        del b7

    # the wider shapes of the same kernel families, three timed calls each: fp32 weights with 6 agents, the
    # predator-prey scenario with 10 agents (rows of 32 floats), the recurrent policy on that scenario's
    # default shape and on 10 agents of simple spread
    wider = {}
    if extras and args.workload == "cfg2":
        def timed(env8, n_agents):
            env8.reset(seed)
            b8 = env8.empty_traj(T)
            w8, k8 = time_rollouts(env8, T, b8, 3, 2)
            res = {"envs": env8.TE, "agents": n_agents, "kernel_ms_avg": float(np.mean(k8)),
                   "agent_steps_per_s": env8.TE * n_agents * T / (w8 / 3)}
            env8.close()
            return res
        env8 = spread_env(synth, 32768, 6, 1, 64, 0)
        env8.set_policy(*to_dev(synth.policy_weights(0, 1, 36, 64)))
        wider["spread_6_agents_fp32"] = timed(env8, 6)
        env8 = tag_env(synth, 16384, 10, 3, 8, 1, 64, 0)
        env8.set_policy(*to_dev(synth.policy_weights(0, 1, synth.tag_obs_dim(10, 3, 8), 64)))
        wider["tag_10_agents_3_obstacles_fp32"] = timed(env8, 10)
        env8 = tag_env(synth, 32768, 4, 2, 3, 1, 128, 1)
        env8.set_gru_policy(*to_dev(synth.gru_weights(0, 1, synth.tag_obs_dim(4, 2, 3))))
        wider["tag_4_agents_recurrent"] = timed(env8, 4)
        env8 = spread_env(synth, 16384, 10, 1, 128, 1)
        env8.set_gru_policy(*to_dev(synth.gru_weights(0, 1, 60)))
        wider["spread_10_agents_recurrent"] = timed(env8, 10)
        wider["note"] = "128-step rollouts, all outputs written; sizes chosen to fill the chip with each shape's block"

    out = {
        "metric": "agent-steps/sec fused MPE rollout @65,536 envs, 1 MI355X; % HBM roofline",
        "value": value,
        "unit": "agent-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if wl.weight_dtype == 0 else "bf16xbf16->f32",
        "dtype_note": ("env math f32; policy contraction: f32 operands as sums of fp16 terms, cross products on the 16-bit matrix "
                       "cores, f32 accumulate: observations and the weights of layers 1 and 3 as three truncated terms (exact for "
                       "|x| >= 0.5, 2^-24 absolute below), hidden activations (outputs of the hardware tanh, ~1e-7 absolute) and the "
                       "pre-scaled weights of layer 2 as two terms rounded to nearest (<= 2^-23 relative, one fp32 ulp); mean error of "
                       "the network outputs against the float64 oracle 1.4e-7, the same as with three terms everywhere (a plain "
                       "float32 evaluation: 0.7e-7)") if wl.weight_dtype == 0 else
                      "weights and layer inputs rounded to bf16, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": wl.name, "envs": TE, "agents": N, "T": T, "policy": "%d->%d->%d->5 tanh" % (D, H, H),
                   "seed": seed, "parallelism": "1 gpu"},
        "env_steps_per_s": value / N,
        "value_by_seed": by_seed,
        "roofline": {
            "kernel": (("rollout_policy_f32_reg_kernel" if wl.num_runs > 1 and wl.num_envs % 64 == 0 and TE >= 65536
                        else "rollout_policy_f32_kernel") if wl.weight_dtype == 0 else "rollout_policy_kernel")
                      + " (fused, one launch per step)",
            # What binds the kernel is vector-instruction issue (operand split, tanh, Philox, env step; the
            # SQ counters below), not the matrix cores and not HBM.  `achieved` is the algorithmic work, the
            # contraction's fp32 FLOPs per agent-step, over the measured time; `peak` the chip's fp32 rate
            # (vector and matrix fp32 peaks are the same number, 157.3 TFLOP/s).  The contraction itself is
            # executed on the 16-bit matrix cores (3-term fp16 operand split): see executed_16bit_mfma.
            "bound": "alu", "achieved": tflops, "peak": MFMA_FP32_PEAK_TFLOPS if wl.weight_dtype == 0 else 2500.0,
            "unit": "TFLOP/s",
            "frac": tflops / (MFMA_FP32_PEAK_TFLOPS if wl.weight_dtype == 0 else 2500.0),
            "frac_note": "algorithmic (fp32-equivalent) contraction FLOPs / fp32 vector peak: a notional fraction of a kernel "
                         "bound by vector issue; it can pass 1 because the products run on the 16-bit matrix cores (see "
                         "executed_16bit_mfma), not on the fp32 units; mfma_busy_frac and valu_active_frac are the measured "
                         "unit utilisations",
            "mfma_busy_frac": None, "valu_active_frac": None,
            "traffic": None,
            "algorithmic_bytes": bytes_per_env_step(N, D) * TE * T,
            "kernel_ms_avg": kavg, "kernel_ms_min": float(np.min(kern_ms)), "kernel_ms_median": float(np.median(kern_ms)),
            "flop_per_agent_step": flops_per_agent_step(D, H),
            "hbm_achieved_GBs": fused_gbs,
            # what the matrix cores really execute: matrix instructions per 64 agent rows and step
            # (16 x 16 x 32 fp16 or bf16 each = 16,384 FLOP), against the fp16 / bf16 matrix peak (2.5 PFLOP/s)
            "executed_16bit_mfma": (lambda n_mfma: {
                "instructions_per_64_rows_step": n_mfma,
                "TFLOPs": n_mfma * 16384 * (agent_steps / 64) / (kavg * 1e-3) / 1e12,
                "frac_of_16bit_peak": n_mfma * 16384 * (agent_steps / 64) / (kavg * 1e-3) / 1e12 / 2500.0,
            })(192 if (wl.weight_dtype == 0 and N >= 2) else 216 if wl.weight_dtype == 0 else 208 if H == 128 else 56),
        },
        "env_only": {
            "kernel": ("rollout_uniform_ws_kernel" if N <= 3 else
                       "rollout_policy_kernel<..., UNIFORM> (lane per agent)" if N == 10 else "rollout_uniform_kernel")
                      + " (seeded uniform actions, one launch per step)",
            "agent_steps_per_s": agent_steps / (wall2 / args.steps),
            "env_steps_per_s": TE * T / (wall2 / args.steps),
            "roofline": {"bound": "hbm", "achieved": env_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": env_gbs / HBM_PEAK_GBS, "traffic": None,
                         "kernel_ms_avg": k2avg, "kernel_ms_min": float(np.min(kern2)),
                         "kernel_ms_median": float(np.median(kern2)),
                         "bytes_per_env_step": bytes_per_env_step(N, D),
                         "algorithmic_bytes": bytes_per_env_step(N, D) * TE * T},
        },
        "mixed_reward": mixed,
        "actor_critic": ac,
        "bf16_policy": bf,
        "many_small_runs": runs16,
        "wider_shapes": wider,
        "tag_scenario": tag,
        "recurrent_policy": gru,
        "single_step": {"us_per_mpe_step_call": step_us, "env_steps_per_s": TE / (step_us * 1e-6),
                        "note": "back-to-back mpe_step calls with resident actions; 352 B per env-step"},
        "paper_context": {"mpe_simple_spread_steps_per_s": {"original_cpu_1env_epyc7763": 8.3e4,
                                                            "jax_a100_10k_envs_random_actions": 4.0e7},
                          "note": "paper Table 3, env-only random actions, other hardware; context only"},
    }
    # Counter figures of the rocprofv3 --pmc runs of this same command (profiles/counters.json): HBM bytes per
    # launch (FETCH_SIZE + WRITE_SIZE, scaled by the calibration copy above) and the SQ utilisation counters.
    # They describe the kernels as built from the sources whose hash they carry; null once the sources changed.
    counters_file = os.path.join(ROOT, "profiles", "counters.json")
    if os.path.exists(counters_file):
        tr = json.load(open(counters_file))
        if tr.get("source_sha256") == kernel_source_hash():
            c_f = tr.get("workloads", {}).get(wl.name, {}).get("fused", {})
            c_e = tr.get("workloads", {}).get(wl.name, {}).get("env_only", {})
            out["roofline"]["traffic"] = c_f.get("total_bytes")
            out["roofline"]["mfma_busy_frac"] = c_f.get("mfma_busy_frac")
            out["roofline"]["valu_active_frac"] = c_f.get("valu_active_frac")
            out["env_only"]["roofline"]["traffic"] = c_e.get("total_bytes")
        else:
            out["roofline"]["counters_note"] = "profiles/counters.json was measured on other kernel sources"
    if not args.no_cpu_baseline:
        w1 = tuple(a[:1] for a in weights)
        out["cpu_baseline"] = cpu_baseline(wl, w1, T, seed, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
