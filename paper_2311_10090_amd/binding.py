"""Thin ctypes binding of libmpe.so (include/mpe.h).  Argument marshalling only.

PyTorch is used for device memory and the current HIP stream; every step of the rollout
runs inside the library's kernels.  There is no CPU fallback: if the library is missing
or the device is absent, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, fields

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpe.so")

MPE_OK, MPE_EINVAL, MPE_ESTATE, MPE_EHIP = 0, -1, -2, -3
WEIGHTS_FP32, WEIGHTS_BF16 = 0, 1
REWARD_SHARED, REWARD_MIXED = 0, 1
SCENARIO_SPREAD, SCENARIO_TAG = 0, 1
NUM_ACTIONS = 5

EXPORTS = ("mpe_create", "mpe_destroy", "mpe_obs_dim", "mpe_reset", "mpe_step", "mpe_set_policy",
           "mpe_rollout", "mpe_set_critic", "mpe_rollout_ac", "mpe_get_state", "mpe_set_state",
           "mpe_set_gru_policy", "mpe_set_gru_critic", "mpe_get_hidden", "mpe_set_hidden", "mpe_rollout_noalloc",
           "mpe_set_barrier_poll_limit", "mpe_last_error")
GRU_HIDDEN = 128


class MpeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libmpe error %d: %s" % (code, msg))
        self.code = code


class _CConfig(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in ("num_envs", "num_agents", "num_landmarks", "num_runs",
                                          "max_episode_steps")] +
                [(n, C.c_float) for n in ("dt", "damping", "mass", "accel", "agent_radius",
                                          "landmark_radius", "contact_force", "contact_margin")] +
                [("hidden", C.c_int32), ("weight_dtype", C.c_int32), ("reward_mode", C.c_int32),
                 ("local_ratio", C.c_float), ("scenario", C.c_int32), ("num_adversaries", C.c_int32)] +
                [(n, C.c_float) for n in ("adv_radius", "adv_accel", "adv_max_speed", "good_max_speed")])


@dataclass
class MpeConfig:
    num_envs: int = 64
    num_agents: int = 3
    num_landmarks: int = 3
    num_runs: int = 1
    max_episode_steps: int = 25
    dt: float = 0.1
    damping: float = 0.25
    mass: float = 1.0
    accel: float = 5.0
    agent_radius: float = 0.15
    landmark_radius: float = 0.05
    contact_force: float = 100.0
    contact_margin: float = 1e-3
    hidden: int = 0
    weight_dtype: int = WEIGHTS_FP32
    reward_mode: int = REWARD_SHARED
    local_ratio: float = 0.5
    scenario: int = SCENARIO_SPREAD
    num_adversaries: int = 0        # SCENARIO_TAG: agents 0..num_adversaries-1; agent_radius / accel: good agents
    adv_radius: float = 0.075
    adv_accel: float = 3.0
    adv_max_speed: float = 1.0
    good_max_speed: float = 1.3

    def to_c(self) -> _CConfig:
        return _CConfig(**{f.name: getattr(self, f.name) for f in fields(self)})


_lib = None


def load_library():
    """Load libmpe.so built in-tree (python -m paper_2311_10090_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libmpe.so is not built: run `python -m paper_2311_10090_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.mpe_last_error.restype = C.c_char_p
    lib.mpe_create.argtypes = [C.POINTER(_CConfig), C.POINTER(vp)]
    lib.mpe_destroy.argtypes = [vp]
    lib.mpe_obs_dim.argtypes = [vp]
    lib.mpe_reset.argtypes = [vp, C.c_uint32, vp, vp]
    lib.mpe_step.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.mpe_set_policy.argtypes = [vp] + [vp] * 6 + [vp]
    lib.mpe_rollout.argtypes = [vp, C.c_int32, vp, vp, vp, vp, vp, vp]
    lib.mpe_get_state.argtypes = [vp, vp, vp, vp, vp, C.POINTER(C.c_uint32), vp]
    lib.mpe_set_state.argtypes = [vp, vp, vp, vp, vp, C.c_uint32, C.c_uint32, vp]
    lib.mpe_set_gru_policy.argtypes = [vp] + [vp] * 10 + [vp]
    lib.mpe_set_gru_critic.argtypes = [vp] + [vp] * 4 + [vp]
    lib.mpe_get_hidden.argtypes = [vp, vp, vp]
    lib.mpe_set_hidden.argtypes = [vp, vp, vp]
    lib.mpe_set_barrier_poll_limit.argtypes = [vp, C.c_uint32]
    lib.mpe_set_critic.argtypes = [vp] + [vp] * 6 + [vp]
    lib.mpe_rollout_ac.argtypes = [vp, C.c_int32] + [vp] * 9
    lib.mpe_rollout_noalloc.argtypes = [C.POINTER(_CConfig), C.c_uint32] + [vp] * 6 + [C.c_int32] + [vp] * 6
    for n in EXPORTS:
        if n != "mpe_last_error":
            getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc < 0:
        raise MpeError(rc, load_library().mpe_last_error().decode())
    return rc


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    if dtype is not None:
        assert t.dtype == dtype, "expected %s, got %s" % (dtype, t.dtype)
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class MpeEnv:
    """Handle around mpe_create/mpe_destroy; methods mirror the C entry points one to one."""

    def __init__(self, cfg: MpeConfig, device="cuda:0"):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.h = C.c_void_p()
        with torch.cuda.device(self.device):
            cc = cfg.to_c()
            _check(self.lib.mpe_create(C.byref(cc), C.byref(self.h)))
        self.E, self.N, self.R, self.L = cfg.num_envs, cfg.num_agents, cfg.num_runs, cfg.num_landmarks
        self.TE = self.E * self.R
        self.D = _check(self.lib.mpe_obs_dim(self.h))
        # rewards per env: one shared value, or one per agent in the mixed mode and in the tag scenario
        per_agent = cfg.reward_mode == REWARD_MIXED or cfg.scenario == SCENARIO_TAG
        self.rew_shape = (self.TE, self.N) if per_agent else (self.TE,)

    def close(self):
        if getattr(self, "h", None) is not None and self.h.value:
            self.lib.mpe_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- allocation helpers (torch is the allocator, nothing else)
    def empty_obs(self, T=None):
        shape = (self.TE, self.N, self.D) if T is None else (T, self.TE, self.N, self.D)
        return torch.empty(shape, dtype=torch.float32, device=self.device)

    def empty_traj(self, T):
        return (self.empty_obs(T),
                torch.empty((T, self.TE, self.N), dtype=torch.uint8, device=self.device),
                torch.empty((T,) + self.rew_shape, dtype=torch.float32, device=self.device),
                torch.empty((T, self.TE), dtype=torch.uint8, device=self.device),
                self.empty_obs())

    # -- entry points
    def reset(self, seed: int, obs=None):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_reset(self.h, seed, _ptr(obs, torch.float32), _stream()))
        return obs

    def step(self, actions, obs=None, reward=None, done=None):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_step(self.h, _ptr(actions, torch.uint8), _ptr(obs, torch.float32),
                                     _ptr(reward, torch.float32), _ptr(done, torch.uint8), _stream()))
        return obs, reward, done

    def set_policy(self, W1=None, b1=None, W2=None, b2=None, W3=None, b3=None):
        args = [_ptr(a, torch.float32) for a in (W1, b1, W2, b2, W3, b3)]
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_policy(self.h, *args, _stream()))

    def rollout(self, T: int, obs_traj=None, act_traj=None, rew_traj=None, done_traj=None, last_obs=None):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_rollout(self.h, T, _ptr(obs_traj, torch.float32), _ptr(act_traj, torch.uint8),
                                        _ptr(rew_traj, torch.float32), _ptr(done_traj, torch.uint8),
                                        _ptr(last_obs, torch.float32), _stream()))
        return obs_traj, act_traj, rew_traj, done_traj, last_obs

    def set_critic(self, V1=None, c1=None, V2=None, c2=None, V3=None, c3=None):
        args = [_ptr(a, torch.float32) for a in (V1, c1, V2, c2, V3, c3)]
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_critic(self.h, *args, _stream()))

    def empty_traj_ac(self, T):
        """obs, act, logp, value, rew, done, last_obs, last_value buffers of mpe_rollout_ac."""
        obs, act, rew, done, last = self.empty_traj(T)
        per_agent = lambda *lead: torch.empty(lead + (self.TE, self.N), dtype=torch.float32, device=self.device)
        return obs, act, per_agent(T), per_agent(T), rew, done, last, per_agent()

    def rollout_ac(self, T: int, obs_traj=None, act_traj=None, logp_traj=None, value_traj=None, rew_traj=None,
                   done_traj=None, last_obs=None, last_value=None):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_rollout_ac(self.h, T, _ptr(obs_traj, torch.float32), _ptr(act_traj, torch.uint8),
                                           _ptr(logp_traj, torch.float32), _ptr(value_traj, torch.float32),
                                           _ptr(rew_traj, torch.float32), _ptr(done_traj, torch.uint8),
                                           _ptr(last_obs, torch.float32), _ptr(last_value, torch.float32), _stream()))
        return obs_traj, act_traj, logp_traj, value_traj, rew_traj, done_traj, last_obs, last_value

    def set_gru_policy(self, *arrays):
        """We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo device tensors (or nothing to remove the policy)."""
        arrays = arrays if arrays else (None,) * 10
        assert len(arrays) == 10
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_gru_policy(self.h, *[_ptr(a, torch.float32) for a in arrays], _stream()))

    def set_gru_critic(self, *arrays):
        """Wc, bc, wv, bv device tensors (or nothing to remove the head)."""
        arrays = arrays if arrays else (None,) * 4
        assert len(arrays) == 4
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_gru_critic(self.h, *[_ptr(a, torch.float32) for a in arrays], _stream()))

    def get_hidden(self):
        h = torch.empty((self.TE, self.N, GRU_HIDDEN), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_get_hidden(self.h, _ptr(h), _stream()))
        return h

    def set_hidden(self, hidden=None):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_hidden(self.h, _ptr(hidden, torch.float32), _stream()))

    def set_barrier_poll_limit(self, polls):
        """Failure-handling hook (see include/mpe.h): 0 restores the default."""
        _check(self.lib.mpe_set_barrier_poll_limit(self.h, int(polls)))

    def get_state(self):
        """Returns pos_a, vel_a ([2][N][TE]), pos_l ([2][L][TE] fp32), ep_step ([TE] int32) tensors and abs_step."""
        pos_a = torch.empty((2, self.N, self.TE), dtype=torch.float32, device=self.device)
        vel_a = torch.empty_like(pos_a)
        pos_l = torch.empty((2, self.L, self.TE), dtype=torch.float32, device=self.device)
        ep = torch.empty((self.TE,), dtype=torch.int32, device=self.device)
        s = C.c_uint32()
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_get_state(self.h, _ptr(pos_a), _ptr(vel_a), _ptr(pos_l), _ptr(ep), C.byref(s), _stream()))
        return pos_a, vel_a, pos_l, ep, int(s.value)

    def set_state(self, pos_a, vel_a, pos_l, ep_step, seed: int, abs_step: int):
        with torch.cuda.device(self.device):
            _check(self.lib.mpe_set_state(self.h, _ptr(pos_a, torch.float32), _ptr(vel_a, torch.float32),
                                          _ptr(pos_l, torch.float32), _ptr(ep_step, torch.int32), seed, abs_step,
                                          _stream()))


def rollout_noalloc(cfg: MpeConfig, seed: int, weights=None, T: int = 1, obs_traj=None, act_traj=None, rew_traj=None,
                    done_traj=None, last_obs=None, device="cuda:0"):
    """mpe_rollout_noalloc: reset(seed) + policy (six device tensors, or None for uniform actions) + T fused
    steps in one call that allocates no device memory; outputs as MpeEnv.rollout."""
    lib = load_library()
    w = [_ptr(a, torch.float32) for a in (weights if weights is not None else (None,) * 6)]
    assert len(w) == 6
    with torch.cuda.device(torch.device(device)):
        cc = cfg.to_c()
        _check(lib.mpe_rollout_noalloc(C.byref(cc), seed, *w, T, _ptr(obs_traj, torch.float32),
                                       _ptr(act_traj, torch.uint8), _ptr(rew_traj, torch.float32),
                                       _ptr(done_traj, torch.uint8), _ptr(last_obs, torch.float32), _stream()))
    return obs_traj, act_traj, rew_traj, done_traj, last_obs
