"""Seeded synthetic inputs and workload shapes.  Holds none of the method's arithmetic.

This is the one module that both the HIP path's callers and the oracle's callers may use:
it only draws numbers from numpy's PCG64 and names the benchmark shapes.  Initial
environment states are NOT made here (both sides derive them from their own Philox);
the arrays below are plain inputs that are handed to either side.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

NUM_ACTIONS = 5

# Physical constants of the simple-spread workload (float32 values are what both sides see).
PHYSICS = dict(dt=0.1, damping=0.25, mass=1.0, accel=5.0, agent_radius=0.15, landmark_radius=0.05,
               contact_force=100.0, contact_margin=1e-3)
MAX_EPISODE_STEPS = 25

# Predator-prey ("simple tag") workload: good agents' radius / gain in agent_radius / accel.
TAG_PHYSICS = dict(dt=0.1, damping=0.25, mass=1.0, accel=4.0, agent_radius=0.05, landmark_radius=0.2,
                   contact_force=100.0, contact_margin=1e-3, adv_radius=0.075, adv_accel=3.0,
                   adv_max_speed=1.0, good_max_speed=1.3)


@dataclass(frozen=True)
class Workload:
    name: str
    num_envs: int          # envs per run
    num_agents: int        # = num_landmarks
    num_runs: int
    T: int
    hidden: int            # 0: no policy (seeded uniform actions)
    weight_dtype: int      # 0 fp32, 1 bf16

    @property
    def obs_dim(self) -> int:
        return 6 * self.num_agents

    @property
    def total_envs(self) -> int:
        return self.num_envs * self.num_runs


WORKLOADS = {
    # small parity case: no policy, uniform actions from the seed
    "cfg0": Workload("cfg0_64env_n3_uniform", 64, 3, 1, 100, 0, 0),
    # fused rollout with the paper's MPE policy shape (two tanh layers of width 64)
    "cfg1": Workload("cfg1_4096env_n3_mlp64_fp32", 4096, 3, 1, 128, 64, 0),
    # headline throughput shape
    "cfg2": Workload("cfg2_65536env_n3_mlp64_fp32", 65536, 3, 1, 128, 64, 0),
    "cfg2_env": Workload("cfg2_65536env_n3_uniform", 65536, 3, 1, 128, 0, 0),
    # scaled scenario, bf16 weights
    "cfg3": Workload("cfg3_16384env_n10_mlp128_bf16", 16384, 10, 1, 128, 128, 1),
    # vectorised independent runs, per-run weights
    "cfg4": Workload("cfg4_1024runs_x64env_n3_mlp64_fp32", 64, 3, 1024, 128, 64, 0),
}


def physics_f32(table=None) -> dict:
    """The constants rounded to float32 and widened again: the exact values the fp32 path uses."""
    return {k: float(np.float32(v)) for k, v in (PHYSICS if table is None else table).items()}


def spread_config(num_envs, num_agents, num_runs=1, hidden=0, weight_dtype=0, max_episode_steps=MAX_EPISODE_STEPS,
                  reward_mode=0, local_ratio=0.5, as_f32=False, **phys) -> dict:
    """Field values of a simple-spread configuration (plain data: keyword arguments for either side's
    config type).  as_f32: the constants rounded to float32 and widened again, i.e. the exact values
    the fp32 path computes with, for a side that takes doubles."""
    p = dict(PHYSICS)
    p.update(phys)
    if as_f32:
        p = {k: float(np.float32(v)) for k, v in p.items()}
        local_ratio = float(np.float32(local_ratio))
    return dict(num_envs=num_envs, num_agents=num_agents, num_landmarks=num_agents, num_runs=num_runs,
                max_episode_steps=max_episode_steps, hidden=hidden, weight_dtype=weight_dtype,
                reward_mode=reward_mode, local_ratio=local_ratio, **p)


def tag_obs_dim(num_agents, num_landmarks, num_adversaries) -> int:
    return 4 + 2 * num_landmarks + 2 * (num_agents - 1) + 2 * (num_agents - num_adversaries)


def tag_config(num_envs, num_agents=4, num_landmarks=2, num_adversaries=3, num_runs=1, hidden=0, weight_dtype=0,
               max_episode_steps=MAX_EPISODE_STEPS, as_f32=False, **phys) -> dict:
    """Field values of a predator-prey configuration: the first num_adversaries agents are adversaries,
    the landmarks are obstacles.  `scenario` is the predator-prey scenario's number on both sides."""
    p = dict(TAG_PHYSICS)
    p.update(phys)
    if as_f32:
        p = {k: float(np.float32(v)) for k, v in p.items()}
    return dict(num_envs=num_envs, num_agents=num_agents, num_landmarks=num_landmarks, num_runs=num_runs,
                max_episode_steps=max_episode_steps, hidden=hidden, weight_dtype=weight_dtype, scenario=1,
                num_adversaries=num_adversaries, **p)


def policy_weights(seed: int, num_runs: int, obs_dim: int, hidden: int):
    """Per-run MLP weights, N(0, 1/fan_in), zero biases, float32.

    Layouts: W1[R][D][H], b1[R][H], W2[R][H][H], b2[R][H], W3[R][H][5], b3[R][5]
    (row-major [fan_in][fan_out]).  Run r uses PCG64(seed + r).
    """
    W1 = np.empty((num_runs, obs_dim, hidden), np.float32)
    W2 = np.empty((num_runs, hidden, hidden), np.float32)
    W3 = np.empty((num_runs, hidden, NUM_ACTIONS), np.float32)
    for r in range(num_runs):
        g = np.random.Generator(np.random.PCG64(seed + r))
        W1[r] = g.standard_normal((obs_dim, hidden)) / np.sqrt(obs_dim)
        W2[r] = g.standard_normal((hidden, hidden)) / np.sqrt(hidden)
        W3[r] = g.standard_normal((hidden, NUM_ACTIONS)) / np.sqrt(hidden)
    b1 = np.zeros((num_runs, hidden), np.float32)
    b2 = np.zeros((num_runs, hidden), np.float32)
    b3 = np.zeros((num_runs, NUM_ACTIONS), np.float32)
    return W1, b1, W2, b2, W3, b3


def policy_weights_with_bias(seed: int, num_runs: int, obs_dim: int, hidden: int):
    """As policy_weights, but with non-zero biases U(-0.5, 0.5) so a dropped bias shows."""
    W1, b1, W2, b2, W3, b3 = policy_weights(seed, num_runs, obs_dim, hidden)
    g = np.random.Generator(np.random.PCG64(seed + 7919))
    b1 = g.uniform(-0.5, 0.5, b1.shape).astype(np.float32)
    b2 = g.uniform(-0.5, 0.5, b2.shape).astype(np.float32)
    b3 = g.uniform(-0.5, 0.5, b3.shape).astype(np.float32)
    return W1, b1, W2, b2, W3, b3


def critic_weights(seed: int, num_runs: int, obs_dim: int, hidden: int):
    """Per-run critic weights (same shape as the policy, one output), N(0, 1/fan_in), biases
    U(-0.5, 0.5), float32: V1[R][D][H], c1[R][H], V2[R][H][H], c2[R][H], V3[R][H], c3[R]."""
    V1 = np.empty((num_runs, obs_dim, hidden), np.float32)
    V2 = np.empty((num_runs, hidden, hidden), np.float32)
    V3 = np.empty((num_runs, hidden), np.float32)
    for r in range(num_runs):
        g = np.random.Generator(np.random.PCG64(seed + 104729 + r))
        V1[r] = g.standard_normal((obs_dim, hidden)) / np.sqrt(obs_dim)
        V2[r] = g.standard_normal((hidden, hidden)) / np.sqrt(hidden)
        V3[r] = g.standard_normal(hidden) / np.sqrt(hidden)
    g = np.random.Generator(np.random.PCG64(seed + 15485863))
    c1 = g.uniform(-0.5, 0.5, (num_runs, hidden)).astype(np.float32)
    c2 = g.uniform(-0.5, 0.5, (num_runs, hidden)).astype(np.float32)
    c3 = g.uniform(-0.5, 0.5, (num_runs,)).astype(np.float32)
    return V1, c1, V2, c2, V3, c3


GRU_HIDDEN = 128


def gru_weights(seed: int, num_runs: int, obs_dim: int):
    """Recurrent-policy weights (hidden 128), N(0, 1/fan_in), biases U(-0.5, 0.5), float32:
    We[R][D][G], be[R][G], Wi[R][G][3G], bi[R][3G], Wh[R][G][3G], bh[R][3G], Wf[R][G][G], bf[R][G],
    Wo[R][G][5], bo[R][5]; gate columns ordered r | z | n."""
    G, R = GRU_HIDDEN, num_runs
    g = np.random.Generator(np.random.PCG64(seed + 32452843))
    mat = lambda fi, fo: (g.standard_normal((R, fi, fo)) / np.sqrt(fi)).astype(np.float32)
    vec = lambda n: g.uniform(-0.5, 0.5, (R, n)).astype(np.float32)
    return (mat(obs_dim, G), vec(G), mat(G, 3 * G), vec(3 * G), mat(G, 3 * G), vec(3 * G), mat(G, G), vec(G),
            mat(G, NUM_ACTIONS), vec(NUM_ACTIONS))


def gru_critic_weights(seed: int, num_runs: int):
    """Critic head of the recurrent actor-critic, float32: Wc[R][G][G] N(0, 1/G), bc[R][G] U(-0.5, 0.5),
    wv[R][G] N(0, 1/G), bv[R] U(-0.5, 0.5)."""
    G, R = GRU_HIDDEN, num_runs
    g = np.random.Generator(np.random.PCG64(seed + 49979687))
    return ((g.standard_normal((R, G, G)) / np.sqrt(G)).astype(np.float32), g.uniform(-0.5, 0.5, (R, G)).astype(np.float32),
            (g.standard_normal((R, G)) / np.sqrt(G)).astype(np.float32), g.uniform(-0.5, 0.5, (R,)).astype(np.float32))


def random_actions(seed: int, shape) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(seed))
    return g.integers(0, NUM_ACTIONS, size=shape, dtype=np.uint8)


def random_state(seed: int, total_envs: int, num_agents: int, num_landmarks: int,
                 max_episode_steps: int = MAX_EPISODE_STEPS, crowded: bool = False):
    """Arbitrary (not reset-generated) float32-representable states for teacher-forced tests.

    crowded=True draws agent positions in a small box so that most pairs are in contact.
    Returns pos_a [TE][N][2], vel_a [TE][N][2], pos_l [TE][L][2] (float32) and ep_step [TE] int32.
    """
    g = np.random.Generator(np.random.PCG64(seed))
    span = 0.25 if crowded else 1.0
    pos_a = g.uniform(-span, span, (total_envs, num_agents, 2)).astype(np.float32)
    vel_a = g.uniform(-1.5, 1.5, (total_envs, num_agents, 2)).astype(np.float32)
    pos_l = g.uniform(-1.0, 1.0, (total_envs, num_landmarks, 2)).astype(np.float32)
    ep = g.integers(0, max_episode_steps, size=total_envs, dtype=np.int32)
    return pos_a, vel_a, pos_l, ep
