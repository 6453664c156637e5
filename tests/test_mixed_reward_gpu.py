"""Parity of the mixed per-agent reward (MPE_REWARD_MIXED) against the oracle, through the C ABI,
for every kernel that writes rewards: mpe_step, the env-only rollout, and both fused rollouts.

The overlap count of an agent is an integer decided by a floating-point comparison (centre
distance below 2 r).  Positions agree with the oracle to ~1e-7 only, so an agent whose distance
to another one lies within 1e-5 of the threshold (in the oracle) is left out of the comparison;
everywhere else the count must be the oracle's, i.e. the reward within the single-step bar."""
import numpy as np
import pytest

from tests import helpers as Hp
from paper_2311_10090_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RATIO = 0.5
TWO_R = 2 * synth.PHYSICS["agent_radius"]


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.fail("gpu tests need a device; the library has no CPU fallback")
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    return MpeEnv, Oracle


def say(msg):
    print(msg, flush=True)


def _pair(mods, E, N, R=1, H=0, wd=0, ratio=RATIO, wseed=None):
    MpeEnv, Oracle = mods
    env = MpeEnv(Hp.gpu_config(E, N, R, H, wd, reward_mode=1, local_ratio=ratio))
    orc = Oracle(Hp.oracle_config(E, N, R, H, wd, reward_mode=1, local_ratio=ratio), threads=8)
    if wseed is not None:
        w = synth.policy_weights_with_bias(wseed, R, 6 * N, H)
        env.set_policy(*Hp.to_dev(w))
        orc.set_policy(*w)
    return env, orc


def _unambiguous(post_pos):
    """[TE][N] bool: no other agent within 1e-5 of the overlap threshold (oracle positions)."""
    d = np.linalg.norm(post_pos[:, :, None, :] - post_pos[:, None, :, :], axis=3)
    n = d.shape[1]
    d[:, np.arange(n), np.arange(n)] = np.inf
    return (np.abs(d - TWO_R) > 1e-5).all(axis=2)


def _forced_steps(env, orc, seed, T, how, crowded_seed=None):
    """Before every step the oracle's state is forced into the library; both then do one step
    (`how` = 'step': mpe_step with random actions; 'rollout': one fused/uniform rollout step)."""
    E, N = env.TE, env.N
    orc.reset(seed)
    env.reset(seed)
    if crowded_seed is not None:
        pa, va, pl, ep = synth.random_state(crowded_seed, E, N, N, crowded=True)
        orc.set_state(pa.astype(np.float64), va.astype(np.float64), pl.astype(np.float64), np.minimum(ep, 3), seed, 0)
    compared = overlapping = 0
    worst = 0.0
    for t in range(T):
        pa, va, pl, ep, s = orc.get_state()
        env.set_state(*Hp.state_to_gpu(pa, va, pl, ep), seed, s)
        if how == "step":
            act = synth.random_actions(100 + t, (E, N))
            robs, rrew, rdone = orc.step(act)
            obs, rew, done = env.step(torch.from_numpy(act).cuda(), env.empty_obs(),
                                      torch.empty(env.rew_shape, dtype=torch.float32, device="cuda"),
                                      torch.empty(E, dtype=torch.uint8, device="cuda"))
            rew, done = rew.cpu().numpy(), done.cpu().numpy()
            ok_env = np.ones(E, bool)
        else:
            robs, ract, rrew, rdone, rlast = orc.rollout(1)
            obs, act, rew, done, last = [x.cpu().numpy() for x in env.rollout(1, *env.empty_traj(1))]
            rew, rrew, done, rdone = rew[0], rrew[0], done[0], rdone[0]
            ok_env = (act[0] == ract[0]).all(axis=1)
        assert rew.shape == (E, N)
        assert np.array_equal(done, rdone)
        live = ok_env & (rdone == 0)                 # after a reset the state holds the new episode
        post = orc.get_state()[0]
        mask = _unambiguous(post) & live[:, None]
        scale = Hp.step_scale(pa)[:, None] * np.ones((1, N))
        worst = max(worst, Hp.assert_close_step(rew[mask], rrew[mask], "mixed reward t=%d" % t, scale[mask]))
        compared += int(mask.sum())
        # how many compared agents really had an overlap (the term under test)
        d = np.linalg.norm(post[:, :, None, :] - post[:, None, :, :], axis=3)
        overlapping += int((((d < TWO_R).sum(axis=2) - 1) > 0)[mask].sum())
    return compared, overlapping, worst


@pytest.mark.parametrize("E,N", [(64, 3), (200, 3), (33, 1), (70, 2), (37, 5), (130, 10)])
def test_step_mixed_reward(mods, E, N):
    say("mixed reward, mpe_step E=%d N=%d" % (E, N))
    env, orc = _pair(mods, E, N)
    compared, overlapping, worst = _forced_steps(env, orc, 5, 6, "step", crowded_seed=17)
    say("  %d agent-steps compared, %d of them overlapping; worst %.2e" % (compared, overlapping, worst))
    assert compared > 0.9 * 6 * E * N and (N == 1 or overlapping > 0.05 * compared)
    env.close()


@pytest.mark.parametrize("E,N,R", [(64, 3, 1), (100, 3, 1), (128, 2, 2), (70, 10, 1), (50, 7, 2), (40, 6, 1), (33, 9, 1)])
def test_uniform_rollout_mixed_reward(mods, E, N, R):
    say("mixed reward, env-only rollout E=%d N=%d R=%d" % (E, N, R))
    env, orc = _pair(mods, E, N, R)
    compared, overlapping, worst = _forced_steps(env, orc, 8, 6, "rollout", crowded_seed=23)
    say("  %d agent-steps compared, %d overlapping; worst %.2e" % (compared, overlapping, worst))
    assert compared > 0.9 * 6 * E * R * N and overlapping > 0.05 * compared
    env.close()


@pytest.mark.parametrize("E,N,R,H,wd", [(256, 3, 1, 64, 0), (100, 2, 1, 64, 0), (64, 3, 3, 64, 0),
                                        (100, 10, 1, 128, 1), (200, 3, 1, 64, 1), (100, 5, 1, 64, 0), (64, 7, 2, 64, 0), (64, 10, 1, 64, 0)])
def test_fused_rollout_mixed_reward(mods, E, N, R, H, wd):
    say("mixed reward, fused rollout E=%d N=%d R=%d H=%d dtype=%d" % (E, N, R, H, wd))
    env, orc = _pair(mods, E, N, R, H, wd, wseed=4)
    compared, overlapping, worst = _forced_steps(env, orc, 9, 6, "rollout", crowded_seed=31)
    say("  %d agent-steps compared, %d overlapping; worst %.2e" % (compared, overlapping, worst))
    assert compared > 0.85 * 6 * E * R * N and overlapping > 0.05 * compared
    env.close()


@pytest.mark.parametrize("N,H,wd", [(3, 0, 0), (3, 64, 0), (10, 128, 1)])
def test_mixed_reward_time_slots_and_ratio_zero(mods, N, H, wd):
    """One rollout of T steps equals T rollouts of one step bit for bit (each reward lands in the
    slot of its own step, across an episode end), and with local_ratio 0 every agent gets the
    shared-mode reward."""
    MpeEnv, _ = mods
    E, T = 96, 28
    w = Hp.to_dev(synth.policy_weights_with_bias(6, 1, 6 * N, H)) if H else None
    envs = [MpeEnv(Hp.gpu_config(E, N, 1, H, wd, reward_mode=1, local_ratio=RATIO)) for _ in range(2)]
    zero = MpeEnv(Hp.gpu_config(E, N, 1, H, wd, reward_mode=1, local_ratio=0.0))
    shared = MpeEnv(Hp.gpu_config(E, N, 1, H, wd))
    for e in envs + [zero, shared]:
        if w:
            e.set_policy(*w)
        e.reset(2)
    full = envs[0].rollout(T, *envs[0].empty_traj(T))
    one = envs[1].empty_traj(1)
    for t in range(T):
        envs[1].rollout(1, *one)
        for k in range(4):
            assert torch.equal(full[k][t], one[k][0]), "output %d at t=%d" % (k, t)
    assert bool(full[3][24].all())
    rz = zero.rollout(T, *zero.empty_traj(T))[2]
    rs = shared.rollout(T, *shared.empty_traj(T))[2]
    assert torch.equal(rz, rs[:, :, None].expand(-1, -1, N))
    # overlaps cost exactly local_ratio each: (shared * (1 - ratio) - mixed) / ratio is a small integer
    cnt = ((1 - RATIO) * rs[:, :, None].double() - full[2].double()) / RATIO
    assert bool(((cnt - cnt.round()).abs() < 1e-5).all()) and cnt.min() > -0.5 and cnt.max() <= N - 1 + 0.5
    for e in envs + [zero, shared]:
        e.close()
