"""Parity at the benchmark's full sizes and launch configurations, on sampled env ranges the
oracle can compute one by one (it simulates envs [offset, offset + n) of run r of the big job),
plus properties that hold at any size."""
import numpy as np
import pytest

from tests import helpers as Hp
from paper_2311_10090_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(msg):
    print(msg, flush=True)


def _gpu_rollout(wl, seed, with_policy=True, wseed=0):
    from paper_2311_10090_amd.binding import MpeEnv
    H = wl.hidden if with_policy else 0
    env = MpeEnv(Hp.gpu_config(wl.num_envs, wl.num_agents, wl.num_runs, H, wl.weight_dtype if with_policy else 0))
    weights = None
    if with_policy:
        weights = synth.policy_weights_with_bias(wseed, wl.num_runs, wl.obs_dim, wl.hidden)
        env.set_policy(*Hp.to_dev(weights))
    env.reset(seed)
    out = env.rollout(wl.T, *env.empty_traj(wl.T))
    torch.cuda.synchronize()
    return env, out, weights


def _make_oracle_range(wl, run, off, n, weights, with_policy=True):
    """Factory of oracles that simulate envs [off, off + n) of run `run` of the big job."""
    from oracle import Oracle
    H = wl.hidden if with_policy else 0

    def make():
        orc = Oracle(Hp.oracle_config(n, wl.num_agents, 1, H, wl.weight_dtype if with_policy else 0,
                                      env_offset=off, run_offset=run), threads=8)
        if with_policy:
            orc.set_policy(*[w[run:run + 1] for w in weights])
        return orc
    return make


class _Sampled:
    """Free-running comparison of sampled env ranges of one big job, pooled: every compared episode is held
    to the 25-step bar over all of its steps (helpers.assert_episodes_close), the sampled actions to their
    agreement bar."""

    def __init__(self, wl, out, seed):
        self.wl, self.out, self.seed = wl, out, seed
        self.err, self.sens, self.gap = [], [], []
        self.agree = self.total = 0

    def add(self, g0, n, make_oracle, what):
        wl, T = self.wl, self.wl.T
        obs, act, rew, done = [x[:, g0:g0 + n].cpu().numpy() for x in self.out[:4]]
        orc = make_oracle()
        orc.reset(self.seed)
        robs, ract, rrew, rdone, rlast = orc.rollout(T)
        assert np.array_equal(done, rdone), what
        for t0 in range(0, T, synth.MAX_EPISODE_STEPS):
            assert np.array_equal(obs[t0].astype(np.float64), robs[t0]), "%s: episode start at t=%d not bit-exact" % (what, t0)
        last = self.out[4][g0:g0 + n].cpu().numpy()
        if T % synth.MAX_EPISODE_STEPS == 0:
            assert np.array_equal(last.astype(np.float64), rlast), "%s: last_obs after a reset not bit-exact" % what
        err, _, (agree, total) = Hp.episode_errors(obs, act, rew, robs, ract, rrew, last=last, rlast=rlast)
        self.err.append(err)
        self.sens.append(Hp.oracle_sensitivity(make_oracle, self.seed, T))
        self.gap.append(Hp.min_gap_spread(robs, wl.num_agents))
        self.agree += agree
        self.total += total

    def check(self, what):
        err, sens, gap = [np.concatenate(x, axis=1) for x in (self.err, self.sens, self.gap)]
        Hp.assert_episodes_close(err, sens, gap, Hp.EXCEED_SHARE_SPREAD[self.wl.num_agents],
                                 what="%s (%d sampled envs)" % (what, err.shape[1]))
        return self.agree / max(self.total, 1), self.total


# Env ranges of a 65,536-env job: the first and the last envs, ranges that straddle 64-env sync groups, 256-env
# blocks (multiples of 256) and the env ranges of two XCDs (multiples of 8,192: blocks are dealt to the eight
# XCDs so that each owns one contiguous eighth of the envs), a single env, odd offsets.  1,093 envs in all.
HEADLINE_RANGES = ((0, 64), (20, 3), (224, 64), (8192 - 32, 64), (12345, 1), (16384 - 100, 200), (24576 - 1, 2),
                   (32736, 64), (40960 - 128, 256), (49152 - 7, 71), (57344 - 64, 128), (61000, 112), (65536 - 64, 64))


@pytest.mark.parametrize("key", ["cfg2", "cfg2_env"])
def test_headline_shape_sampled_against_oracle(key):
    wl = synth.WORKLOADS[key]
    with_policy = wl.hidden > 0
    say("full size %s: %d envs x %d steps" % (wl.name, wl.total_envs, wl.T))
    env, out, weights = _gpu_rollout(wl, seed=1, with_policy=with_policy, wseed=3)
    obs, act, rew, done, last = out
    # properties at full size
    assert int(done.sum().item()) == wl.total_envs * (wl.T // synth.MAX_EPISODE_STEPS)
    assert bool((done[24::25] == 1).all())
    assert bool((obs[..., 14:] == 0).all()), "comm slots must be zero"
    assert bool((act <= 4).all()) and bool(torch.isfinite(obs).all()) and bool((rew <= 0).all())
    hist = torch.bincount(act.flatten().long(), minlength=5).double()
    assert hist.min() > 0.02 * hist.sum()
    samp = _Sampled(wl, out, 1)
    assert sum(n for _, n in HEADLINE_RANGES) >= 1024
    for off, n in HEADLINE_RANGES:
        samp.add(off, n, _make_oracle_range(wl, 0, off, n, weights, with_policy), "%s envs %d..%d" % (key, off, off + n))
    frac, tot = samp.check("full size %s" % wl.name)
    say("  sampled action agreement %.6f over %d samples" % (frac, tot))
    if with_policy:
        assert frac >= Hp.ACTION_AGREEMENT - 2.0 / tot
    else:
        assert frac == 1.0  # uniform actions are integer work
    env.close()


def test_per_run_weights_full_size():
    """1,024 runs x 64 envs: the launch of 256-env blocks whose four sync groups hold the weights of four
    different runs and whose rows live in registers.  Sampled runs against the oracle; run 0 must also
    equal, bit for bit, a single-run job with that run's weights (the 64-env block kernel with its LDS
    observation tile: same arithmetic, another data path)."""
    from paper_2311_10090_amd.binding import MpeEnv
    wl = synth.WORKLOADS["cfg4"]
    say("full size %s: %d runs x %d envs" % (wl.name, wl.num_runs, wl.num_envs))
    env, out, weights = _gpu_rollout(wl, seed=1, wseed=11)
    # 40 of the 1,024 runs: the four runs of the first and of the last 256-env block, runs on either side of an
    # XCD's range of blocks (128 runs each), and a stride through the rest
    runs = sorted(set([0, 1, 2, 3, 127, 128, 129, 511, 512, 517, 895, 896, 1020, 1021, 1022, 1023] + list(range(37, 1024, 41))))
    assert len(runs) >= 32
    samp = _Sampled(wl, out, 1)
    for run in runs:
        samp.add(run * 64, 64, _make_oracle_range(wl, run, 0, 64, weights), "run %d" % run)
    frac, tot = samp.check("full size %s" % wl.name)
    say("  sampled action agreement %.6f over %d samples" % (frac, tot))
    assert frac >= Hp.ACTION_AGREEMENT - 2.0 / tot
    one = MpeEnv(Hp.gpu_config(64, wl.num_agents, 1, wl.hidden, 0))
    one.set_policy(*Hp.to_dev([w[0:1] for w in weights]))
    one.reset(1)
    ref0 = one.rollout(wl.T, *one.empty_traj(wl.T))
    for k in range(4):
        assert torch.equal(out[k][:, :64], ref0[k]), "run 0, output %d" % k
    assert torch.equal(out[4][:64], ref0[4])
    one.close()
    env.close()


@pytest.mark.parametrize("N,R,E", [(2, 1024, 64), (3, 1023, 64), (3, 512, 128)])
def test_per_run_weights_other_shapes_full_size(N, R, E):
    """Two agents; a batch whose last 256-env block is ragged (1,023 runs: three groups and an empty one);
    runs of 128 envs (two sync groups of a block share a run)."""
    wl = synth.Workload("runs_%dx%denv_n%d_mlp64_fp32" % (R, E, N), E, N, R, 60, 64, 0)
    say("full size %s" % wl.name)
    env, out, weights = _gpu_rollout(wl, seed=2, wseed=12)
    assert int(out[3].sum().item()) == wl.total_envs * (wl.T // synth.MAX_EPISODE_STEPS)
    assert bool(torch.isfinite(out[0]).all()) and bool((out[1] <= 4).all())
    samp = _Sampled(wl, out, 2)
    for run in (0, 1, 5, R // 2, R - 3, R - 2, R - 1):
        samp.add(run * E + E - 64, 64, _make_oracle_range(wl, run, E - 64, 64, weights), "run %d" % run)
    frac, tot = samp.check("full size %s" % wl.name)
    say("  sampled action agreement %.6f over %d samples" % (frac, tot))
    assert frac >= Hp.ACTION_AGREEMENT - 2.0 / tot
    s = env.get_state()
    assert bool(torch.isfinite(s[0]).all()) and int(s[4]) == wl.T
    env.close()


def test_wide_bf16_full_size():
    wl = synth.WORKLOADS["cfg3"]
    say("full size %s: %d envs x %d agents" % (wl.name, wl.total_envs, wl.num_agents))
    env, out, weights = _gpu_rollout(wl, seed=1, wseed=5)
    obs, act, rew, done, last = out
    assert int(done.sum().item()) == wl.total_envs * (wl.T // synth.MAX_EPISODE_STEPS)
    assert bool((obs[..., 42:] == 0).all()) and bool(torch.isfinite(obs).all())
    # 288 envs: first and last, ranges across 32-env sync groups, 64-env blocks and the XCDs' ranges (2,048 envs)
    samp = _Sampled(wl, out, 1)
    for off, n in ((0, 32), (48, 32), (2048 - 16, 32), (8176, 32), (10240 - 40, 64), (12288 + 31, 34), (wl.num_envs - 62, 62)):
        samp.add(off, n, _make_oracle_range(wl, 0, off, n, weights), "cfg3 envs %d..%d" % (off, off + n))
    frac, tot = samp.check("full size %s" % wl.name)
    say("  bf16 sampled action agreement %.5f over %d samples (no bar)" % (frac, tot))
    assert frac >= 0.99
    env.close()


def test_large_ragged_size_uses_256_env_blocks():
    """A single run a little over 65,536 envs: the fused kernel runs 256-env blocks of four sync
    groups, the last block holds 74 valid envs (one full group, one group of 10, two empty)."""
    wl = synth.Workload("ragged_65610env_n3_mlp64_fp32", 65610, 3, 1, 60, 64, 0)
    say("full size %s" % wl.name)
    env, out, weights = _gpu_rollout(wl, seed=2, wseed=7)
    obs, act, rew, done, last = out
    assert int(done.sum().item()) == wl.total_envs * (wl.T // synth.MAX_EPISODE_STEPS)
    assert bool(torch.isfinite(obs).all()) and bool((act <= 4).all())
    samp = _Sampled(wl, out, 2)
    for off, n in ((65536 - 40, 40), (65536, 64), (65600, 10), (300, 20), (8192 - 10, 20)):
        samp.add(off, n, _make_oracle_range(wl, 0, off, n, weights), "ragged envs %d..%d" % (off, off + n))
    frac, tot = samp.check("full size %s" % wl.name)
    say("  sampled action agreement %.6f over %d samples" % (frac, tot))
    assert frac >= Hp.ACTION_AGREEMENT - 2.0 / tot
    # same job through the actor-critic entry point (also 256-env blocks): identical plain outputs
    env2, _, _ = _gpu_rollout(wl, seed=2, wseed=7)
    env2.set_critic(*Hp.to_dev(synth.critic_weights(7, 1, wl.obs_dim, wl.hidden)))
    env2.reset(2)
    ac = env2.rollout_ac(wl.T, *env2.empty_traj_ac(wl.T))
    for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
        assert torch.equal(ac[k_ac], out[k_pl])
    assert bool(torch.isfinite(ac[2]).all()) and bool(torch.isfinite(ac[3]).all()) and bool(torch.isfinite(ac[7]).all())
    env.close()
    env2.close()


@pytest.mark.parametrize("N", [1, 2])
def test_large_size_one_and_two_agents_use_256_env_blocks(N):
    """65,600 envs with 1 and 2 agents: the fused kernel's 256-env blocks (four sync groups of N
    wavefronts, each group on one SIMD), sampled env ranges against the oracle."""
    wl = synth.Workload("large_65600env_n%d_mlp64_fp32" % N, 65600, N, 1, 50, 64, 0)
    say("full size %s" % wl.name)
    env, out, weights = _gpu_rollout(wl, seed=4, wseed=8)
    assert int(out[3].sum().item()) == wl.total_envs * (wl.T // synth.MAX_EPISODE_STEPS)
    assert bool(torch.isfinite(out[0]).all()) and bool((out[1] <= 4).all())
    samp = _Sampled(wl, out, 4)
    for off, n in ((0, 64), (255, 130), (32768 - 30, 64), (65536, 64)):
        samp.add(off, n, _make_oracle_range(wl, 0, off, n, weights), "N=%d envs %d..%d" % (N, off, off + n))
    frac, tot = samp.check("full size %s" % wl.name)
    say("  sampled action agreement %.6f over %d samples" % (frac, tot))
    assert frac >= Hp.ACTION_AGREEMENT - 2.0 / tot
    env.close()


def _compare_mixed_rewards(outs, ref, g0, n, N, T, what):
    """Rewards on the first steps of each episode, for envs whose actions so far agree, leaving out agents
    within 1e-4 of the overlap threshold; episode starts bit-exact.  Returns the number compared."""
    obs, act, rew = outs[0], outs[1], outs[2]
    robs, ract, rrew, rdone, rlast = ref
    a = act[:, g0:g0 + n].cpu().numpy()
    r = rew[:, g0:g0 + n].cpu().numpy()
    o = obs[:, g0:g0 + n].cpu().numpy()
    compared = 0
    for t0 in (0, 25):
        for t in range(t0, min(t0 + 4, T - 1)):
            alive = (a[t0:t + 1] == ract[t0:t + 1]).all(axis=(0, 2))
            # positions after step t = own-position entries of the next observation (no reset inside)
            pos = robs[t + 1][:, :, 2:4]
            d = np.linalg.norm(pos[:, :, None, :] - pos[:, None, :, :], axis=3)
            d[:, np.arange(N), np.arange(N)] = np.inf
            mask = (np.abs(d - 0.3) > 1e-4).all(axis=2) & alive[:, None]
            assert np.abs(r[t][mask] - rrew[t][mask]).max() <= Hp.EPISODE_ATOL, "%s, t=%d" % (what, t)
            compared += int(mask.sum())
    assert np.array_equal(o[0].astype(np.float64), robs[0]) and np.array_equal(o[25].astype(np.float64), robs[25]), what
    return compared


def test_large_size_mixed_reward():
    """Mixed per-agent reward through the 256-env block path, sampled against the oracle."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    E, N, T = 65610, 3, 30
    say("full size mixed reward: %d envs" % E)
    w = synth.policy_weights_with_bias(5, 1, 18, 64)
    env = MpeEnv(Hp.gpu_config(E, N, 1, 64, 0, reward_mode=1, local_ratio=0.5))
    env.set_policy(*Hp.to_dev(w))
    env.reset(3)
    outs = env.rollout(T, *env.empty_traj(T))
    assert outs[2].shape == (T, E, N)
    compared = 0
    for off, n in ((0, 64), (65536 - 20, 40), (65600, 10), (40000, 64)):
        orc = Oracle(Hp.oracle_config(n, N, 1, 64, 0, env_offset=off, reward_mode=1, local_ratio=0.5), threads=8)
        orc.set_policy(*w)
        orc.reset(3)
        compared += _compare_mixed_rewards(outs, orc.rollout(T), off, n, N, T, "envs %d.." % off)
    say("  %d agent rewards compared" % compared)
    assert compared > 3000
    env.close()


def test_per_run_weights_mixed_reward_full_size():
    """1,024 runs x 64 envs with the mixed per-agent reward (the register-row launch): sampled runs against
    the oracle, and run 0 bit for bit against a single-run job with that run's weights."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    E, N, R, T = 64, 3, 1024, 30
    say("full size mixed reward, %d runs x %d envs" % (R, E))
    w = synth.policy_weights_with_bias(6, R, 18, 64)
    env = MpeEnv(Hp.gpu_config(E, N, R, 64, 0, reward_mode=1, local_ratio=0.5))
    env.set_policy(*Hp.to_dev(w))
    env.reset(4)
    outs = env.rollout(T, *env.empty_traj(T))
    assert outs[2].shape == (T, E * R, N)
    compared = 0
    for run in (0, 3, 514, R - 1):
        orc = Oracle(Hp.oracle_config(E, N, 1, 64, 0, run_offset=run, reward_mode=1, local_ratio=0.5), threads=8)
        orc.set_policy(*[x[run:run + 1] for x in w])
        orc.reset(4)
        compared += _compare_mixed_rewards(outs, orc.rollout(T), run * E, E, N, T, "run %d" % run)
    say("  %d agent rewards compared" % compared)
    assert compared > 3000
    one = MpeEnv(Hp.gpu_config(E, N, 1, 64, 0, reward_mode=1, local_ratio=0.5))
    one.set_policy(*Hp.to_dev([x[0:1] for x in w]))
    one.reset(4)
    ref0 = one.rollout(T, *one.empty_traj(T))
    for k in range(4):
        assert torch.equal(outs[k][:, :E], ref0[k]), "run 0, output %d" % k
    assert torch.equal(outs[4][:E], ref0[4])
    one.close()
    env.close()


# ------------------------------------------------------------------ second scenario, full size
@pytest.mark.parametrize("with_policy", [True, False])
def test_tag_scenario_full_size(with_policy):
    """Predator-prey at the bench's size (65,536 envs x 4 agents x 128 steps, the launch bench.py
    times), sampled env ranges against the oracle plus properties of the whole trajectory."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    E, T, shape = 65536, 128, (4, 2, 3)
    N, L, A = shape
    H = 64 if with_policy else 0
    say("full size tag scenario, policy=%s" % with_policy)
    env = MpeEnv(Hp.tag_gpu_config(E, N, L, A, 1, H))
    w = synth.policy_weights_with_bias(3, 1, env.D, 64) if with_policy else None
    if w:
        env.set_policy(*Hp.to_dev(w))
    env.reset(1)
    obs, act, rew, done, last = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    assert int(done.sum().item()) == E * (T // 25) and bool((done[24::25] == 1).all())
    assert bool((act <= 4).all()) and bool(torch.isfinite(obs).all()) and bool(torch.isfinite(rew).all())
    assert bool((obs[:, :, 3, 14:] == 0).all()), "the good agent's row ends with two zeros"
    assert bool((rew[:, :, :3] >= 0).all()) and bool((rew[:, :, 3] <= 0).all())
    assert bool((rew[:, :, 0] == rew[:, :, 1]).all()) and bool((rew[:, :, 0] == rew[:, :, 2]).all())
    adv = rew[:, :, 0]
    assert bool(((adv / 10 - (adv / 10).round()).abs() < 1e-6).all()) and float(adv.max()) >= 10.0
    speed = obs[..., 0:2].norm(dim=-1)
    assert float(speed[:, :, :3].max()) <= 1.0 + 1e-5 and float(speed[:, :, 3].max()) <= 1.3 + 1e-5
    tot = agree = 0
    errs, senss, gaps = [], [], []
    # 519 envs: first and last, ranges across 64-env blocks and the XCDs' ranges (8,192 envs), an odd offset
    for off, n in ((0, 64), (8192 - 32, 64), (16384 + 40, 48), (32741, 7), (40960 - 64, 128), (57344 - 72, 144), (E - 64, 64)):
        def make_oracle(off=off, n=n):
            o_ = Oracle(Hp.tag_oracle_config(n, N, L, A, 1, H, env_offset=off), threads=8)
            if w:
                o_.set_policy(*w)
            return o_
        orc = make_oracle()
        orc.reset(1)
        robs, ract, rrew, rdone, rlast = orc.rollout(T)
        o, a, r, d = [x[:, off:off + n].cpu().numpy() for x in (obs, act, rew, done)]
        assert np.array_equal(d, rdone)
        err, _, (ag, to) = Hp.episode_errors(o, a, None, robs, ract, None, last=last[off:off + n].cpu().numpy(), rlast=rlast)
        agree += ag
        tot += to
        errs.append(err)
        senss.append(Hp.oracle_sensitivity(make_oracle, 1, T))
        gaps.append(Hp.min_gap_tag(robs, shape))
        for t0 in range(0, T, 25):
            alive = np.logical_and.accumulate((a[t0:t0 + 25] == ract[t0:t0 + 25]).all(axis=2), axis=0)
            # rewards of the first steps of an episode (same positions to 1e-4: same touching decisions
            # unless a pair sits on the threshold, which these few samples do not)
            assert (np.abs(r[t0:t0 + 5] - rrew[t0:t0 + 5]).max(axis=2) * alive[:5]).max() <= 1e-3
    err, sens, gap = [np.concatenate(x, axis=1) for x in (errs, senss, gaps)]
    Hp.assert_episodes_close(err, sens, gap, Hp.EXCEED_SHARE_TAG[shape[:2]],
                             what="full size tag scenario, policy=%s (%d sampled envs)" % (with_policy, err.shape[1]))
    say("  sampled action agreement %.6f over %d samples" % (agree / tot, tot))
    assert (agree / tot >= Hp.ACTION_AGREEMENT - 2.0 / tot) if with_policy else agree == tot
    env.close()


def test_tag_actor_critic_full_size():
    """The predator-prey actor-critic rollout at the bench's size (65,536 envs: 512 blocks of 128 envs):
    plain outputs bit-identical to mpe_rollout's, log-probabilities and values of sampled env ranges
    against the oracle's networks on the recorded observations."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    from scipy.special import log_softmax
    E, T, shape = 65536, 64, (4, 2, 3)
    N, L, A = shape
    say("full size tag actor-critic")
    a, b = MpeEnv(Hp.tag_gpu_config(E, N, L, A, 1, 64)), MpeEnv(Hp.tag_gpu_config(E, N, L, A, 1, 64))
    D = a.D
    pw, cw = synth.policy_weights_with_bias(3, 1, D, 64), synth.critic_weights(3, 1, D, 64)
    for env in (a, b):
        env.set_policy(*Hp.to_dev(pw))
        env.reset(1)
    a.set_critic(*Hp.to_dev(cw))
    full = a.rollout_ac(T, *a.empty_traj_ac(T))
    plain = b.rollout(T, *b.empty_traj(T))
    torch.cuda.synchronize()
    for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
        assert torch.equal(full[k_ac], plain[k_pl]), "output %d differs from mpe_rollout" % k_ac
    assert bool(torch.isfinite(full[2]).all()) and bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all())
    orc = Oracle(Hp.tag_oracle_config(64, N, L, A, 1, 64), threads=8)
    orc.set_policy(*pw)
    orc.set_critic(*cw)
    for off, n in ((0, 128), (32700, 100), (E - 128, 128)):
        rows = full[0][:, off:off + n].cpu().numpy().reshape(-1, D).astype(np.float64)
        act = full[1][:, off:off + n].cpu().numpy().reshape(-1)
        ref_lp = log_softmax(orc.policy_logits(rows), axis=1)[np.arange(rows.shape[0]), act]
        Hp.assert_close_step(full[2][:, off:off + n].cpu().numpy().reshape(-1), ref_lp, "log-prob")
        Hp.assert_close_step(full[3][:, off:off + n].cpu().numpy().reshape(-1), orc.value(rows), "value")
        last_rows = full[6][off:off + n].cpu().numpy().reshape(-1, D).astype(np.float64)
        Hp.assert_close_step(full[7][off:off + n].cpu().numpy().reshape(-1), orc.value(last_rows), "bootstrap value")
    a.close()
    b.close()


# ------------------------------------------------------------------ recurrent policy, full size
def test_recurrent_policy_full_size():
    """GRU policy at the bench's size (65,536 envs x 3 agents x 128 steps): sampled env ranges against
    the oracle (bf16 network: actions agree while no rounding flip has changed a sample; >= 99 %)."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    E, T, N = 65536, 128, 3
    say("full size recurrent policy")
    env = MpeEnv(Hp.gpu_config(E, N, 1, 128, 1))
    w = synth.gru_weights(5, 1, 18)
    env.set_gru_policy(*Hp.to_dev(w))
    env.reset(1)
    obs, act, rew, done, last = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    assert int(done.sum().item()) == E * (T // 25) and bool((done[24::25] == 1).all())
    assert bool((act <= 4).all()) and bool(torch.isfinite(obs).all()) and bool((rew <= 0).all())
    hist = torch.bincount(act.flatten().long(), minlength=5).double()
    assert hist.min() > 0.02 * hist.sum()
    hid = env.get_hidden()
    assert bool(torch.isfinite(hid).all()) and float(hid.abs().max()) <= 1.0 and bool(hid.any())
    tot = agree = 0
    errs, senss, gaps = [], [], []
    for off, n in ((0, 64), (8192 - 32, 64), (32741, 7), (49152 - 16, 48), (E - 64, 64)):
        def make_oracle(off=off, n=n):
            o_ = Oracle(Hp.oracle_config(n, N, 1, 128, 1, env_offset=off), threads=8)
            o_.set_gru(*w)
            return o_
        orc = make_oracle()
        orc.reset(1)
        robs, ract, rrew, rdone, rlast = orc.rollout(T)
        o, a, r, d = [x[:, off:off + n].cpu().numpy() for x in (obs, act, rew, done)]
        assert np.array_equal(d, rdone)
        for t0 in range(0, T, 25):
            assert np.array_equal(o[t0].astype(np.float64), robs[t0])
        err, _, (ag, to) = Hp.episode_errors(o, a, r, robs, ract, rrew, last=last[off:off + n].cpu().numpy(), rlast=rlast)
        agree += ag
        tot += to
        errs.append(err)
        senss.append(Hp.oracle_sensitivity(make_oracle, 1, T))
        gaps.append(Hp.min_gap_spread(robs, N))
        # carried state at the end (T = 128: 3 steps into an episode) where the whole last episode agreed
        h = hid[off:off + n].cpu().numpy().astype(np.float64)
        ok = (a[125:] == ract[125:]).all(axis=(0, 2))
        dh = np.abs(h - orc.get_hidden())[ok]
        assert dh.size and np.median(dh) < 1e-5 and dh.max() < 2e-2
    err, sens, gap = [np.concatenate(x, axis=1) for x in (errs, senss, gaps)]
    Hp.assert_episodes_close(err, sens, gap, Hp.EXCEED_SHARE_SPREAD[N],
                             what="full size recurrent policy (%d sampled envs)" % err.shape[1])
    say("  sampled action agreement %.6f over %d samples" % (agree / tot, tot))
    assert agree / tot >= 0.99
    env.close()


def test_recurrent_actor_critic_full_size():
    """Recurrent actor-critic at the bench's size (65,536 envs x 3 agents x 128 steps, the launch shape of
    bench.py's recurrent_policy.actor_critic): plain outputs and carried state bit-identical to mpe_rollout's;
    sampled env ranges against the oracle's actor-critic rollout, episode by episode (every episode starts
    from the same reset state on both sides), on the envs whose sampled actions agree so far."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    E, T, N = 65536, 128, 3
    say("full size recurrent actor-critic")
    w, c = synth.gru_weights(5, 1, 18), synth.gru_critic_weights(5, 1)
    env = MpeEnv(Hp.gpu_config(E, N, 1, 128, 1))
    env.set_gru_policy(*Hp.to_dev(w))
    env.set_gru_critic(*Hp.to_dev(c))
    env.reset(1)
    obs, act, logp, val, rew, done, last, lastv = env.rollout_ac(T, *env.empty_traj_ac(T))
    hid = env.get_hidden()
    plain = MpeEnv(Hp.gpu_config(E, N, 1, 128, 1))
    plain.set_gru_policy(*Hp.to_dev(w))
    plain.reset(1)
    p = plain.rollout(T, *plain.empty_traj(T))
    for got, ref, name in ((obs, p[0], "obs"), (act, p[1], "act"), (rew, p[2], "rew"), (done, p[3], "done"), (last, p[4], "last_obs"),
                           (hid, plain.get_hidden(), "carried state")):
        assert torch.equal(got, ref), name
    plain.close()
    del p
    assert bool((logp <= 0).all()) and bool(torch.isfinite(val).all()) and bool(torch.isfinite(lastv).all())
    ev, el, eb = [], [], []
    for off, n in ((0, 64), (8192 - 16, 32), (32741, 7), (E - 32, 32)):
        orc = Oracle(Hp.oracle_config(n, N, 1, 128, 1, env_offset=off), threads=8)
        orc.set_gru(*w)
        orc.set_gru_critic(*c)
        orc.reset(1)
        robs, ract, rlogp, rval, rrew, rdone, rlast, rlastv = orc.rollout_ac(T)
        a, lp, v = [x[:, off:off + n].cpu().numpy() for x in (act, logp, val)]
        same = (a == ract).all(axis=2)
        for t0 in range(0, T, 25):
            alive = np.logical_and.accumulate(same[t0:t0 + 25], axis=0)
            prior = np.vstack([np.ones((1, n), bool), alive[:-1]])
            ev.append(np.abs(v[t0:t0 + 25] - rval[t0:t0 + 25])[prior])
            el.append(np.abs(lp[t0:t0 + 25] - rlogp[t0:t0 + 25])[alive])
        eb.append(np.abs(lastv[off:off + n].cpu().numpy() - rlastv)[alive[-1]])
    for name, e in (("value", np.concatenate(ev)), ("log-prob", np.concatenate(el)), ("bootstrap value", np.concatenate(eb))):
        say("  %s: median %.2e, mean %.2e, worst %.2e over %d" % (name, np.median(e), e.mean(), e.max(), e.size))
        assert e.size > 100 and np.median(e) < 2e-6 and e.mean() < 5e-4 and e.max() < 5e-2, name
    env.close()


@pytest.mark.parametrize("scn,E,recurrent", [(6, 32768, False), ((10, 3, 8), 16384, False), ((4, 2, 3), 32768, True), (10, 16384, True)])
def test_wider_shapes_at_the_sizes_the_bench_times(scn, E, recurrent):
    """The launches of bench.py's wider_shapes section (fp32 weights with 6 agents, predator-prey with 10 agents,
    the recurrent policy on predator-prey and on 10 agents of simple spread), 128 steps: sampled env ranges
    against the oracle, every episode of the rollout (each starts from a reset state that is the same bits on
    both sides), with the 25-step bar of the small-size tests."""
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    T = 128
    tag = isinstance(scn, tuple)
    H, wd = (128, 1) if recurrent else (64, 0)
    say("full size wider shape scenario=%s E=%d recurrent=%s" % (scn, E, recurrent))
    if tag:
        N, L, A = scn
        env = MpeEnv(Hp.tag_gpu_config(E, N, L, A, 1, H, wd=wd))
    else:
        N = scn
        env = MpeEnv(Hp.gpu_config(E, N, 1, H, wd))
    w = synth.gru_weights(5, 1, env.D) if recurrent else synth.policy_weights_with_bias(3, 1, env.D, 64)
    (env.set_gru_policy if recurrent else env.set_policy)(*Hp.to_dev(w))
    env.reset(1)
    obs, act, rew, done, last = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    assert int(done.sum().item()) == E * (T // 25) and bool((done[24::25] == 1).all())
    assert bool((act <= 4).all()) and bool(torch.isfinite(obs).all()) and bool(torch.isfinite(rew).all())
    tot = agree = 0
    errs, senss, gaps = [], [], []
    for off, n in ((0, 32), (E // 8 - 16, 32), (E // 2 + 5, 7), (E - 32, 32)):
        def make_oracle(off=off, n=n):
            cfg = (Hp.tag_oracle_config(n, N, L, A, 1, H, env_offset=off, wd=wd) if tag
                   else Hp.oracle_config(n, N, 1, H, wd, env_offset=off))
            o_ = Oracle(cfg, threads=8)
            (o_.set_gru if recurrent else o_.set_policy)(*w)
            return o_
        orc = make_oracle()
        orc.reset(1)
        robs, ract, rrew, rdone, rlast = orc.rollout(T)
        o, a, r, d = [x[:, off:off + n].cpu().numpy() for x in (obs, act, rew, done)]
        assert np.array_equal(d, rdone)
        err, _, (ag, to) = Hp.episode_errors(o, a, None if tag else r, robs, ract, None if tag else rrew,
                                              last=last[off:off + n].cpu().numpy(), rlast=rlast)
        agree += ag
        tot += to
        errs.append(err)
        senss.append(Hp.oracle_sensitivity(make_oracle, 1, T))
        gaps.append(Hp.min_gap_tag(robs, scn) if tag else Hp.min_gap_spread(robs, N))
    err, sens, gap = [np.concatenate(x, axis=1) for x in (errs, senss, gaps)]
    share = Hp.EXCEED_SHARE_TAG[scn[:2]] if tag else Hp.EXCEED_SHARE_SPREAD[N]
    Hp.assert_episodes_close(err, sens, gap, share, what="full size wider shape scenario=%s E=%d recurrent=%s (%d sampled envs)" % (scn, E, recurrent, err.shape[1]))
    say("  sampled action agreement %.6f over %d samples" % (agree / tot, tot))
    assert agree / tot >= (0.97 if recurrent else Hp.ACTION_AGREEMENT - 2.0 / tot)
    env.close()
