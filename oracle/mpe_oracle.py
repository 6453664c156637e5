"""ctypes loader for the CPU oracle (oracle/mpe_oracle.cpp).  Test infrastructure only.

Argument marshalling and nothing else: every number comes out of the C++ file.
All arrays are host numpy arrays in the oracle's own plain layouts:
  obs [R*E][N][D] float64, reward [R*E] float64 ([R*E][N] in reward_mode 1 and in scenario 1), done [R*E] uint8,
  actions [R*E][N] uint8,
  pos_a / vel_a [R*E][N][2], pos_l [R*E][L][2] float64, ep_step [R*E] int32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mpe_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
             "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "num_envs", "num_agents", "num_landmarks", "num_runs", "max_episode_steps",
        "hidden", "weight_dtype", "env_offset", "run_offset")] + [(n, C.c_double) for n in (
        "dt", "damping", "mass", "accel", "agent_radius", "landmark_radius",
        "contact_force", "contact_margin")] + [("reward_mode", C.c_int32), ("reserved", C.c_int32),
                                               ("local_ratio", C.c_double),
                                               ("scenario", C.c_int32), ("num_adversaries", C.c_int32)] + [
        (n, C.c_double) for n in ("adv_radius", "adv_accel", "adv_max_speed", "good_max_speed")]


@dataclass
class OracleConfig:
    num_envs: int = 64
    num_agents: int = 3
    num_landmarks: int = 3
    num_runs: int = 1
    max_episode_steps: int = 25
    hidden: int = 64
    weight_dtype: int = 0
    env_offset: int = 0
    run_offset: int = 0
    dt: float = 0.1
    damping: float = 0.25
    mass: float = 1.0
    accel: float = 5.0
    agent_radius: float = 0.15
    landmark_radius: float = 0.05
    contact_force: float = 100.0
    contact_margin: float = 1e-3
    reward_mode: int = 0        # 0: shared coverage reward [R*E]; 1: mixed per-agent reward [R*E][N]
    reserved: int = 0
    local_ratio: float = 0.5
    scenario: int = 0           # 0 simple spread; 1 simple tag (rewards [R*E][N]; agent_radius / accel: good agents)
    num_adversaries: int = 0
    adv_radius: float = 0.075
    adv_accel: float = 3.0
    adv_max_speed: float = 1.0
    good_max_speed: float = 1.3


_lib = None


def _load():
    global _lib
    if _lib is None:
        # MPE_ORACLE_LIB: load another build of the same source instead (the sanitizer and mutation tests
        # compile instrumented or deliberately broken copies into a temporary folder)
        _lib = C.CDLL(os.environ.get("MPE_ORACLE_LIB") or build())
        _lib.orc_last_error.restype = C.c_char_p
        _lib.orc_round_to_bf16.restype = C.c_double
        _lib.orc_round_to_bf16.argtypes = [C.c_double]
        _lib.orc_create.argtypes = [C.POINTER(_CConfig), C.POINTER(C.c_void_p)]
        for name in ("orc_destroy", "orc_obs_dim"):
            getattr(_lib, name).argtypes = [C.c_void_p]
        _lib.orc_set_threads.argtypes = [C.c_void_p, C.c_int]
        _lib.orc_observe.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_reset.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        _lib.orc_step.argtypes = [C.c_void_p] + [C.c_void_p] * 4
        _lib.orc_set_policy.argtypes = [C.c_void_p] + [C.c_void_p] * 6
        _lib.orc_policy_logits.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
        _lib.orc_gumbel_max_action.argtypes = [C.c_uint32] * 5 + [C.c_void_p]
        _lib.orc_uniform_action.argtypes = [C.c_uint32] * 5
        _lib.orc_rollout.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 5
        _lib.orc_get_state.argtypes = [C.c_void_p] + [C.c_void_p] * 5
        _lib.orc_set_state.argtypes = [C.c_void_p] + [C.c_void_p] * 4 + [C.c_uint32, C.c_uint32]
        _lib.orc_philox4x32_10.argtypes = [C.c_void_p] * 3
        _lib.orc_set_critic.argtypes = [C.c_void_p] + [C.c_void_p] * 6
        _lib.orc_value.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
        _lib.orc_log_probs.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_log_probs.restype = None
        _lib.orc_rollout_ac.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 8
        _lib.orc_set_gru.argtypes = [C.c_void_p] + [C.c_void_p] * 10
        _lib.orc_gru_forward.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.orc_set_gru_critic.argtypes = [C.c_void_p] + [C.c_void_p] * 4
        _lib.orc_get_hidden.argtypes = [C.c_void_p, C.c_void_p]
        _lib.orc_set_hidden.argtypes = [C.c_void_p, C.c_void_p]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(rc):
    if rc != 0:
        raise RuntimeError("oracle: " + _load().orc_last_error().decode())


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _load().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def gumbel_max_action(seed, run, env, step, agent, logits) -> int:
    z = np.ascontiguousarray(logits, dtype=np.float64)
    assert z.shape == (5,)
    return int(_load().orc_gumbel_max_action(seed, run, env, step, agent, _ptr(z)))


def uniform_action(seed, run, env, step, agent) -> int:
    return int(_load().orc_uniform_action(seed, run, env, step, agent))


def log_probs(logits) -> np.ndarray:
    z = np.ascontiguousarray(logits, dtype=np.float64)
    assert z.shape == (5,)
    out = np.empty(5, dtype=np.float64)
    _load().orc_log_probs(_ptr(z), _ptr(out))
    return out


def round_to_bf16(x: float) -> float:
    return float(_load().orc_round_to_bf16(float(x)))


class Oracle:
    def __init__(self, cfg: OracleConfig, threads: int = 1):
        self.cfg = cfg
        self.lib = _load()
        cc = _CConfig(**{f[0]: getattr(cfg, f[0]) for f in _CConfig._fields_})
        h = C.c_void_p()
        _check(self.lib.orc_create(C.byref(cc), C.byref(h)))
        self.h = h
        self.E, self.N, self.L, self.R = cfg.num_envs, cfg.num_agents, cfg.num_landmarks, cfg.num_runs
        self.TE = self.E * self.R
        self.D = int(self.lib.orc_obs_dim(self.h))
        self.threads = threads
        self.rew_shape = (self.TE, self.N) if (cfg.reward_mode == 1 or cfg.scenario == 1) else (self.TE,)
        _check(self.lib.orc_set_threads(self.h, threads))

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.orc_destroy(self.h)
            self.h = None

    def reset(self, seed: int) -> np.ndarray:
        obs = np.empty((self.TE, self.N, self.D), dtype=np.float64)
        _check(self.lib.orc_reset(self.h, seed, _ptr(obs)))
        return obs

    def observe(self) -> np.ndarray:
        obs = np.empty((self.TE, self.N, self.D), dtype=np.float64)
        _check(self.lib.orc_observe(self.h, _ptr(obs)))
        return obs

    def step(self, actions: np.ndarray):
        a = np.ascontiguousarray(actions, dtype=np.uint8)
        assert a.shape == (self.TE, self.N)
        obs = np.empty((self.TE, self.N, self.D), dtype=np.float64)
        rew = np.empty(self.rew_shape, dtype=np.float64)
        done = np.empty(self.TE, dtype=np.uint8)
        _check(self.lib.orc_step(self.h, _ptr(a), _ptr(obs), _ptr(rew), _ptr(done)))
        return obs, rew, done

    def set_policy(self, W1, b1, W2, b2, W3, b3):
        if W1 is None:
            _check(self.lib.orc_set_policy(self.h, None, None, None, None, None, None))
            return
        H = self.cfg.hidden
        shapes = [(self.R, self.D, H), (self.R, H), (self.R, H, H), (self.R, H), (self.R, H, 5), (self.R, 5)]
        arrs = []
        for a, s in zip((W1, b1, W2, b2, W3, b3), shapes):
            a = np.ascontiguousarray(a, dtype=np.float32).reshape(s)
            arrs.append(a)
        _check(self.lib.orc_set_policy(self.h, *[_ptr(a) for a in arrs]))

    def set_critic(self, V1, c1, V2, c2, V3, c3):
        """Critic of the actor-critic rollout: same shape as the policy with one output."""
        if V1 is None:
            _check(self.lib.orc_set_critic(self.h, None, None, None, None, None, None))
            return
        H = self.cfg.hidden
        shapes = [(self.R, self.D, H), (self.R, H), (self.R, H, H), (self.R, H), (self.R, H), (self.R,)]
        arrs = [np.ascontiguousarray(a, dtype=np.float32).reshape(s) for a, s in zip((V1, c1, V2, c2, V3, c3), shapes)]
        _check(self.lib.orc_set_critic(self.h, *[_ptr(a) for a in arrs]))

    GRU_H = 128

    def gru_shapes(self):
        G, R, D = self.GRU_H, self.R, self.D
        return [(R, D, G), (R, G), (R, G, 3 * G), (R, 3 * G), (R, G, 3 * G), (R, 3 * G), (R, G, G), (R, G),
                (R, G, 5), (R, 5)]

    def set_gru(self, *arrays):
        """Recurrent policy: We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo (or nothing to remove it)."""
        if not arrays or arrays[0] is None:
            _check(self.lib.orc_set_gru(self.h, *([None] * 10)))
            return
        arrs = [np.ascontiguousarray(a, dtype=np.float32).reshape(s) for a, s in zip(arrays, self.gru_shapes())]
        assert len(arrs) == 10
        _check(self.lib.orc_set_gru(self.h, *[_ptr(a) for a in arrs]))

    def set_gru_critic(self, Wc=None, bc=None, wv=None, bv=None):
        """Critic head of the recurrent actor-critic: Wc [R][128][128], bc [R][128], wv [R][128], bv [R]
        (or nothing to remove it)."""
        if Wc is None:
            _check(self.lib.orc_set_gru_critic(self.h, None, None, None, None))
            return
        G, R = self.GRU_H, self.R
        shapes = [(R, G, G), (R, G), (R, G), (R,)]
        arrs = [np.ascontiguousarray(a, dtype=np.float32).reshape(sh) for a, sh in zip((Wc, bc, wv, bv), shapes)]
        _check(self.lib.orc_set_gru_critic(self.h, *[_ptr(a) for a in arrs]))

    def gru_forward(self, obs_rows, hidden, run: int = 0, with_value: bool = False):
        """One evaluation per row: returns (new hidden [n][128], logits [n][5]) and, with_value, the critic
        head's value [n] of the new hidden state."""
        o = np.ascontiguousarray(obs_rows, dtype=np.float64).reshape(-1, self.D)
        h = np.array(hidden, dtype=np.float64).reshape(o.shape[0], self.GRU_H).copy()
        z = np.empty((o.shape[0], 5), dtype=np.float64)
        v = np.empty(o.shape[0], dtype=np.float64) if with_value else None
        _check(self.lib.orc_gru_forward(self.h, run, _ptr(o), o.shape[0], _ptr(h), _ptr(z), _ptr(v) if with_value else None))
        return (h, z, v) if with_value else (h, z)

    def get_hidden(self) -> np.ndarray:
        h = np.empty((self.TE, self.N, self.GRU_H), dtype=np.float64)
        _check(self.lib.orc_get_hidden(self.h, _ptr(h)))
        return h

    def set_hidden(self, hidden=None):
        if hidden is None:
            _check(self.lib.orc_set_hidden(self.h, None))
        else:
            h = np.ascontiguousarray(hidden, dtype=np.float64).reshape(self.TE, self.N, self.GRU_H)
            _check(self.lib.orc_set_hidden(self.h, _ptr(h)))

    def value(self, obs_rows: np.ndarray, run: int = 0) -> np.ndarray:
        o = np.ascontiguousarray(obs_rows, dtype=np.float64).reshape(-1, self.D)
        out = np.empty(o.shape[0], dtype=np.float64)
        _check(self.lib.orc_value(self.h, run, _ptr(o), o.shape[0], _ptr(out)))
        return out

    def rollout_ac(self, T: int):
        """Returns obs, act, logp, value, rew, done, last_obs, last_value."""
        obs = np.empty((T, self.TE, self.N, self.D), dtype=np.float64)
        act = np.empty((T, self.TE, self.N), dtype=np.uint8)
        logp = np.empty((T, self.TE, self.N), dtype=np.float64)
        val = np.empty((T, self.TE, self.N), dtype=np.float64)
        rew = np.empty((T,) + self.rew_shape, dtype=np.float64)
        done = np.empty((T, self.TE), dtype=np.uint8)
        last = np.empty((self.TE, self.N, self.D), dtype=np.float64)
        lastv = np.empty((self.TE, self.N), dtype=np.float64)
        _check(self.lib.orc_rollout_ac(self.h, T, _ptr(obs), _ptr(act), _ptr(logp), _ptr(val), _ptr(rew),
                                       _ptr(done), _ptr(last), _ptr(lastv)))
        return obs, act, logp, val, rew, done, last, lastv

    def policy_logits(self, obs_rows: np.ndarray, run: int = 0) -> np.ndarray:
        o = np.ascontiguousarray(obs_rows, dtype=np.float64).reshape(-1, self.D)
        out = np.empty((o.shape[0], 5), dtype=np.float64)
        _check(self.lib.orc_policy_logits(self.h, run, _ptr(o), o.shape[0], _ptr(out)))
        return out

    def rollout(self, T: int, want_obs: bool = True):
        obs = np.empty((T, self.TE, self.N, self.D), dtype=np.float64) if want_obs else None
        act = np.empty((T, self.TE, self.N), dtype=np.uint8)
        rew = np.empty((T,) + self.rew_shape, dtype=np.float64)
        done = np.empty((T, self.TE), dtype=np.uint8)
        last = np.empty((self.TE, self.N, self.D), dtype=np.float64)
        _check(self.lib.orc_rollout(self.h, T, _ptr(obs), _ptr(act), _ptr(rew), _ptr(done), _ptr(last)))
        return obs, act, rew, done, last

    def get_state(self):
        pos_a = np.empty((self.TE, self.N, 2), dtype=np.float64)
        vel_a = np.empty((self.TE, self.N, 2), dtype=np.float64)
        pos_l = np.empty((self.TE, self.L, 2), dtype=np.float64)
        ep = np.empty(self.TE, dtype=np.int32)
        s = C.c_uint32()
        _check(self.lib.orc_get_state(self.h, _ptr(pos_a), _ptr(vel_a), _ptr(pos_l), _ptr(ep),
                                      C.cast(C.byref(s), C.c_void_p)))
        return pos_a, vel_a, pos_l, ep, int(s.value)

    def set_state(self, pos_a, vel_a, pos_l, ep_step, seed: int, abs_step: int):
        pa = np.ascontiguousarray(pos_a, dtype=np.float64).reshape(self.TE, self.N, 2)
        va = np.ascontiguousarray(vel_a, dtype=np.float64).reshape(self.TE, self.N, 2)
        pl = np.ascontiguousarray(pos_l, dtype=np.float64).reshape(self.TE, self.L, 2)
        ep = np.ascontiguousarray(ep_step, dtype=np.int32).reshape(self.TE)
        _check(self.lib.orc_set_state(self.h, _ptr(pa), _ptr(va), _ptr(pl), _ptr(ep), seed, abs_step))
