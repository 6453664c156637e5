"""Parity of mpe_rollout_ac (log-probability of the sampled action, critic value, bootstrap value)
against the oracle, through the C ABI.  Bars: actions as in the plain fused rollout; log-prob and
value within 1e-5 * max(1, |ref|) of the oracle on teacher-forced observations; the plain outputs
bit-identical to mpe_rollout's."""
import numpy as np
import pytest

from tests import helpers as Hp
from paper_2311_10090_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.fail("gpu tests need a device; the library has no CPU fallback")
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    return MpeEnv, Oracle


def say(msg):
    print(msg, flush=True)


def _pair(mods, E, N, R=1, wseed=3, wd=0, **kw):
    MpeEnv, Oracle = mods
    env = MpeEnv(Hp.gpu_config(E, N, R, 64, wd, **kw))
    orc = Oracle(Hp.oracle_config(E, N, R, 64, wd, **kw), threads=8)
    pw = synth.policy_weights_with_bias(wseed, R, 6 * N, 64)
    cw = synth.critic_weights(wseed, R, 6 * N, 64)
    env.set_policy(*Hp.to_dev(pw))
    env.set_critic(*Hp.to_dev(cw))
    orc.set_policy(*pw)
    orc.set_critic(*cw)
    return env, orc


@pytest.mark.parametrize("E,N,R,T,wd", [(1024, 3, 1, 30, 0), (300, 3, 1, 30, 0), (100, 2, 1, 20, 0), (70, 1, 1, 20, 0),
                                        (256, 3, 2, 12, 0), (64, 3, 3, 12, 0), (300, 3, 1, 20, 1), (70, 1, 1, 10, 1),
                                        (300, 4, 1, 15, 0), (130, 5, 1, 12, 0), (64, 6, 2, 10, 0), (100, 7, 1, 10, 0), (32, 7, 3, 8, 0),
                                        (100, 8, 1, 8, 0), (16, 9, 3, 8, 0), (70, 10, 1, 8, 0)])
def test_actor_critic_teacher_forced(mods, E, N, R, T, wd):
    """The oracle runs free; before every step its state is forced into the library, which then does
    one actor-critic step.  wd = 1: bf16 weights and layer inputs on both sides."""
    say("actor-critic teacher-forced E=%d N=%d R=%d T=%d dtype=%d" % (E, N, R, T, wd))
    env, orc = _pair(mods, E, N, R, wd=wd)
    orc.reset(13)
    env.reset(13)
    bufs = env.empty_traj_ac(1)
    agree = total = 0
    worst_lp = worst_v = 0.0
    for t in range(T):
        pa, va, pl, ep, s = orc.get_state()
        env.set_state(*Hp.state_to_gpu(pa, va, pl, ep), 13, s)
        robs, ract, rlogp, rval, rrew, rdone, rlast, rlastv = orc.rollout_ac(1)
        obs, act, logp, val, rew, done, last, lastv = [x.cpu().numpy() for x in env.rollout_ac(1, *bufs)]
        Hp.assert_close_step(obs, robs, "obs acted on")
        assert np.array_equal(done, rdone)
        same = act == ract
        agree += int(same.sum())
        total += same.size
        if wd == 0:
            worst_v = max(worst_v, Hp.assert_close_step(val, rval, "value"))
            worst_lp = max(worst_lp, Hp.assert_close_step(logp[same], rlogp[same], "log-prob of the sampled action"))
        else:
            # bf16 layer inputs: where the device's tanh (hardware exp2 and rcp, ~1e-7 absolute) and
            # the oracle's fall on different sides of a bf16 rounding boundary, one hidden unit moves
            # by 2^-8 of its value and an output by ~1e-3; a small hidden value (|h| ~ 1e-2) has
            # boundaries only 2e-5 apart, so a fair share of the outputs carries one such flip.
            # No bar is stated for bf16: most outputs must still meet the fp32 bar, all a loose one.
            for got, ref, what in ((val, rval, "value"), (logp[same], rlogp[same], "log-prob")):
                err = np.abs(got - ref) / np.maximum(1.0, np.abs(ref))
                assert (err <= Hp.STEP_RTOL).mean() >= 0.6 and err.max() < 2e-2 and err.mean() < 1e-3, what
                worst_v = max(worst_v, float(err.max()))
        ok = same.all(axis=2)[0]
        scale = Hp.step_scale(pa)[ok]
        if wd == 0:
            Hp.assert_close_step(lastv[ok], rlastv[ok], "bootstrap value", scale[:, None])
        Hp.assert_close_step(rew[0][ok], rrew[0][ok], "reward", scale)
    say("  action agreement %.6f over %d; worst log-prob error %.2e, value error %.2e" % (agree / total, total, worst_lp, worst_v))
    assert (1.0 - agree / total) * total <= max(2, 1e-4 * total)
    env.close()


@pytest.mark.parametrize("E,N,kw", [(512, 3, {}), (200, 3, dict(reward_mode=1, local_ratio=0.5)), (130, 2, {})])
def test_actor_critic_rollout_matches_plain_rollout_and_itself(mods, E, N, kw):
    """obs, actions, rewards, done and last_obs are bit-identical to mpe_rollout's (the same policy
    arithmetic in another block shape), log-prob and value of step t are functions of obs[t] only
    (checked against the oracle's networks on the recorded observations), T steps = T/2 + T/2."""
    MpeEnv, Oracle = mods
    T = 32
    say("actor-critic free-running E=%d N=%d %s" % (E, N, kw))
    a, orc = _pair(mods, E, N, 1, wseed=9, **kw)
    b, _ = _pair(mods, E, N, 1, wseed=9, **kw)
    c, _ = _pair(mods, E, N, 1, wseed=9, **kw)
    for e in (a, b, c):
        e.reset(21)
    full = a.rollout_ac(T, *a.empty_traj_ac(T))
    plain = b.rollout(T, *b.empty_traj(T))
    for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
        assert torch.equal(full[k_ac], plain[k_pl]), "output %d differs from mpe_rollout" % k_ac
    h1 = [x.clone() for x in c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))]
    h2 = c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))
    for k in range(6):
        assert torch.equal(full[k], torch.cat([h1[k], h2[k]])), "continuation, output %d" % k
    assert torch.equal(full[6], h2[6]) and torch.equal(full[7], h2[7])
    obs, act, logp, val = [x.cpu().numpy() for x in full[:4]]
    rows = obs.reshape(-1, 6 * N).astype(np.float64)
    z = orc.policy_logits(rows)
    from scipy.special import log_softmax
    ref_lp = log_softmax(z, axis=1)[np.arange(z.shape[0]), act.reshape(-1)]
    Hp.assert_close_step(logp.reshape(-1), ref_lp, "log-prob from recorded obs and actions")
    Hp.assert_close_step(val.reshape(-1), orc.value(rows), "value from recorded obs")
    Hp.assert_close_step(full[7].cpu().numpy().reshape(-1),
                         orc.value(full[6].cpu().numpy().reshape(-1, 6 * N).astype(np.float64)), "bootstrap value")
    assert bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all())
    for e in (a, b, c):
        e.close()


def test_actor_critic_errors_and_absent_outputs(mods):
    MpeEnv, _ = mods
    from paper_2311_10090_amd.binding import MpeError, MPE_EINVAL, MPE_ESTATE
    env = MpeEnv(Hp.gpu_config(64, 3, 1, 64, 0))
    env.reset(0)
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2)
    assert ei.value.code == MPE_ESTATE
    env.set_policy(*Hp.to_dev(synth.policy_weights(0, 1, 18, 64)))
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2)
    assert ei.value.code == MPE_ESTATE
    env.set_critic(*Hp.to_dev(synth.critic_weights(0, 1, 18, 64)))
    ref = MpeEnv(Hp.gpu_config(64, 3, 1, 64, 0))
    ref.set_policy(*Hp.to_dev(synth.policy_weights(0, 1, 18, 64)))
    ref.reset(0)
    env.rollout_ac(7)                       # no outputs at all
    ref.rollout(7)
    for x, y in zip(env.get_state(), ref.get_state()):
        assert torch.equal(x, y) if hasattr(x, "shape") else x == y
    env.close()
    ref.close()
    eight = MpeEnv(Hp.gpu_config(64, 8, 1, 128, 0))   # fp32 networks are 64 wide
    with pytest.raises(MpeError) as ei:
        eight.set_critic(*Hp.to_dev(synth.critic_weights(0, 1, 48, 128)))
    assert ei.value.code == MPE_EINVAL
    eight.close()
    runs = MpeEnv(Hp.gpu_config(40, 3, 2, 64, 0))     # several runs need num_envs % 64 == 0
    runs.set_policy(*Hp.to_dev(synth.policy_weights(0, 2, 18, 64)))
    runs.set_critic(*Hp.to_dev(synth.critic_weights(0, 2, 18, 64)))
    runs.reset(0)
    with pytest.raises(MpeError) as ei:
        runs.rollout_ac(2)
    assert ei.value.code == MPE_EINVAL
    runs.close()



@pytest.mark.parametrize("N,H,E,R,kw", [(10, 128, 96, 1, {}), (4, 64, 200, 1, {}), (7, 64, 70, 1, {}), (8, 128, 32, 2, {}),
                                        (6, 64, 64, 2, dict(reward_mode=1, local_ratio=0.5)), (5, 128, 130, 1, {})])
def test_actor_critic_with_four_and_more_agents(mods, N, H, E, R, kw):
    """The lane-per-agent bf16 kernel with a critic: plain outputs bit-identical to mpe_rollout's, T steps =
    T/2 + T/2, log-probabilities and values against the oracle's bf16 networks on the recorded observations
    (the statistical bar of bf16 layer inputs: most outputs within the fp32 bar, all within a loose one)."""
    from scipy.special import log_softmax
    MpeEnv, Oracle = mods
    T, D, TE = 16, 6 * N, E * R
    say("actor-critic N=%d H=%d E=%d R=%d %s" % (N, H, E, R, kw))
    pw = synth.policy_weights_with_bias(19, R, D, H)
    cw = synth.critic_weights(19, R, D, H)

    def make(critic=True):
        e = MpeEnv(Hp.gpu_config(E, N, R, H, 1, **kw))
        e.set_policy(*Hp.to_dev(pw))
        if critic:
            e.set_critic(*Hp.to_dev(cw))
        e.reset(23)
        return e
    a, b, c = make(), make(False), make()
    orc = Oracle(Hp.oracle_config(E, N, R, H, 1, **kw), threads=8)
    orc.set_policy(*pw)
    orc.set_critic(*cw)
    full = a.rollout_ac(T, *a.empty_traj_ac(T))
    plain = b.rollout(T, *b.empty_traj(T))
    for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
        assert torch.equal(full[k_ac], plain[k_pl]), "output %d differs from mpe_rollout" % k_ac
    h1 = [x.clone() for x in c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))]
    h2 = c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))
    for k in range(6):
        assert torch.equal(full[k], torch.cat([h1[k], h2[k]])), "continuation, output %d" % k
    assert torch.equal(full[6], h2[6]) and torch.equal(full[7], h2[7])
    obs, act, logp, val = [x.cpu().numpy() for x in full[:4]]
    last, lastv = full[6].cpu().numpy(), full[7].cpu().numpy()
    assert logp.shape == (T, TE, N) and val.shape == (T, TE, N) and lastv.shape == (TE, N)
    for run in range(R):
        sl = slice(run * E, (run + 1) * E)
        rows = obs[:, sl].reshape(-1, D).astype(np.float64)
        z = orc.policy_logits(rows, run=run)
        ref_lp = log_softmax(z, axis=1)[np.arange(z.shape[0]), act[:, sl].reshape(-1)]
        pairs = ((logp[:, sl].reshape(-1), ref_lp, "log-prob"), (val[:, sl].reshape(-1), orc.value(rows, run=run), "value"),
                 (lastv[sl].reshape(-1), orc.value(last[sl].reshape(-1, D).astype(np.float64), run=run), "bootstrap value"))
        for got, ref, what in pairs:
            err = np.abs(got - ref) / np.maximum(1.0, np.abs(ref))
            say("  run %d %s: within 1e-5 %.3f, mean %.2e, worst %.2e" % (run, what, (err <= Hp.STEP_RTOL).mean(), err.mean(), err.max()))
            assert (err <= Hp.STEP_RTOL).mean() >= 0.9 and err.max() < 2e-2 and err.mean() < 1e-4, what
    assert bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all())
    for e in (a, b, c):
        e.close()


@pytest.mark.parametrize("scn", ["spread", "tag", "spread6"])
def test_fp32_network_outputs_are_as_close_to_float64_as_a_plain_float32_evaluation(mods, scn):
    """The fp32 mode runs its products on the 16-bit matrix cores with operands held as sums of fp16 terms (to
    within one fp32 unit in the last place).  What that costs is measured here on the outputs themselves: over
    hundreds of thousands of recorded rows, values and log-probabilities must lie as close to the oracle's
    float64 networks as a plain float32 evaluation of the same networks does (numpy, correctly rounded tanh),
    up to the error of the hardware tanh (~1e-7 absolute per activation): mean error below 2.5e-7 and at most
    3 times the plain evaluation's, worst error below 3e-6."""
    from scipy.special import log_softmax
    MpeEnv, Oracle = mods
    E, T = 8192, 25
    if scn == "tag":
        gcfg, ocfg = Hp.tag_gpu_config(E, 4, 2, 3, 1, 64), Hp.tag_oracle_config(E, 4, 2, 3, 1, 64)
    else:
        N = 6 if scn == "spread6" else 3
        E = E // (N // 3)
        gcfg, ocfg = Hp.gpu_config(E, N, 1, 64, 0), Hp.oracle_config(E, N, 1, 64, 0)
    env, orc = MpeEnv(gcfg), Oracle(ocfg, threads=8)
    D = env.D
    w, c = synth.policy_weights_with_bias(3, 1, D, 64), synth.critic_weights(3, 1, D, 64)
    env.set_policy(*Hp.to_dev(w))
    env.set_critic(*Hp.to_dev(c))
    orc.set_policy(*w)
    orc.set_critic(*c)
    env.reset(5)
    obs, act, lp, v = [x.cpu().numpy() for x in env.rollout_ac(T, *env.empty_traj_ac(T))[:4]]
    rows = obs.reshape(-1, D)
    rv = orc.value(rows.astype(np.float64))
    rlp = log_softmax(orc.policy_logits(rows.astype(np.float64)), axis=1)[np.arange(rows.shape[0]), act.reshape(-1)]
    ev, el = np.abs(v.reshape(-1) - rv), np.abs(lp.reshape(-1) - rlp)
    V1, c1, V2, c2, V3, c3 = [a[0].astype(np.float32) for a in c]
    h = np.tanh(np.tanh(rows @ V1 + c1) @ V2 + c2)
    plain = np.abs(((h @ V3.reshape(64, -1)).reshape(-1) + c3.reshape(-1)[0]).astype(np.float64) - rv)
    say("  %s: value error mean %.3e worst %.3e, log-prob error mean %.3e worst %.3e over %d rows; plain float32 numpy value error mean %.3e worst %.3e"
        % (scn, ev.mean(), ev.max(), el.mean(), el.max(), ev.size, plain.mean(), plain.max()))
    Hp.record("fp32 network outputs against the float64 oracle, %s, %d rows: value error mean %.3e worst %.3e, log-prob error mean %.3e worst %.3e; "
              "plain float32 numpy evaluation of the value head: mean %.3e worst %.3e" % (scn, ev.size, ev.mean(), ev.max(), el.mean(), el.max(), plain.mean(), plain.max()))
    assert ev.mean() < 2.5e-7 and el.mean() < 2.5e-7 and ev.max() < 3e-6 and el.max() < 3e-6
    assert ev.mean() <= 3.0 * plain.mean()
    env.close()
