"""Actor-critic rollout (mpe_rollout_ac) of the predator-prey scenario against the oracle, through the
C ABI.  The kernel runs the plain fused rollout's policy arithmetic in another block shape (8
wavefronts around two staged networks), so its plain outputs must be bit-identical to mpe_rollout's,
which the scenario's own parity tests hold to the oracle; log-probability and value are compared with
the oracle's networks, teacher-forced and on the recorded observations (1e-5 * max(1, |ref|))."""
import numpy as np
import pytest
from scipy.special import log_softmax

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


def _weights(shape, R, wseed):
    D = Hp.tag_obs_dim(*shape)
    return synth.policy_weights_with_bias(wseed, R, D, 64), synth.critic_weights(wseed, R, D, 64)


def _env(mods, E, shape, R=1, wseed=3, critic=True, wd=0):
    env = mods[0](Hp.tag_gpu_config(E, *shape, R, 64, wd=wd))
    pw, cw = _weights(shape, R, wseed)
    env.set_policy(*Hp.to_dev(pw))
    if critic:
        env.set_critic(*Hp.to_dev(cw))
    return env


def _oracle(mods, E, shape, R=1, wseed=3, wd=0):
    orc = mods[1](Hp.tag_oracle_config(E, *shape, R, 64, wd=wd), threads=8)
    pw, cw = _weights(shape, R, wseed)
    orc.set_policy(*pw)
    orc.set_critic(*cw)
    return orc


def _assert_network_outputs(got, ref, what, wd):
    """fp32 weights: the single-step bar.  bf16 weights and layer inputs: a value that sits on a bf16 rounding
    boundary can round the other way on the fp32 path and move an output by ~1e-3, so most outputs must
    meet the fp32 bar and all a loose one (the bar of the simple-spread bf16 networks)."""
    if wd == 0:
        Hp.assert_close_step(got, ref, what)
        return
    err = np.abs(got - ref) / np.maximum(1.0, np.abs(ref))
    say("  %s: within 1e-5 %.3f, mean %.2e, worst %.2e" % (what, (err <= Hp.STEP_RTOL).mean(), err.mean(), err.max()))
    assert (err <= Hp.STEP_RTOL).mean() >= 0.9 and err.max() < 2e-2 and err.mean() < 1e-4, what


@pytest.mark.parametrize("shape,E,R,wd", [((4, 2, 3), 1024, 1, 0), ((4, 2, 3), 200, 1, 0), ((4, 2, 3), 1, 1, 0), ((4, 2, 3), 129, 1, 0),
                                          ((2, 1, 1), 300, 1, 0), ((2, 1, 1), 256, 1, 0), ((3, 0, 2), 130, 1, 0),
                                          ((4, 2, 3), 128, 3, 0), ((2, 1, 1), 256, 2, 0), ((3, 0, 2), 64, 2, 0),
                                          ((6, 2, 4), 130, 1, 0), ((5, 2, 4), 100, 1, 0), ((8, 2, 6), 64, 2, 0), ((10, 3, 8), 70, 1, 0),
                                          ((6, 2, 4), 16, 3, 0), ((10, 3, 8), 32, 2, 0),
                                          ((4, 2, 3), 200, 1, 1), ((2, 1, 1), 256, 2, 1), ((3, 0, 2), 130, 1, 1), ((6, 2, 4), 100, 1, 1),
                                          ((10, 3, 8), 64, 1, 1), ((4, 2, 3), 16, 4, 1)])
def test_matches_plain_rollout_continues_and_agrees_with_the_oracles_networks(mods, shape, E, R, wd):
    N, T = shape[0], 32
    D = Hp.tag_obs_dim(*shape)
    say("tag actor-critic shape=%s E=%d R=%d dtype=%d" % (shape, E, R, wd))
    a, b, c = (_env(mods, E, shape, R, 9, wd=wd), _env(mods, E, shape, R, 9, critic=False, wd=wd),
               _env(mods, E, shape, R, 9, wd=wd))
    orc = _oracle(mods, E, shape, R, 9, wd=wd)
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
    for x, y in zip(a.get_state(), b.get_state()):
        assert torch.equal(x, y) if hasattr(x, "shape") else x == y
    obs, act, logp, val = [x.cpu().numpy() for x in full[:4]]
    TE = E * R
    for run in range(R):
        sl = slice(run * E, (run + 1) * E)
        rows = obs[:, sl].reshape(-1, D).astype(np.float64)
        z = orc.policy_logits(rows, run=run)
        ref_lp = log_softmax(z, axis=1)[np.arange(z.shape[0]), act[:, sl].reshape(-1)]
        _assert_network_outputs(logp[:, sl].reshape(-1), ref_lp, "log-prob from recorded obs and actions", wd)
        _assert_network_outputs(val[:, sl].reshape(-1), orc.value(rows, run=run), "value from recorded obs", wd)
        last_rows = full[6][sl].cpu().numpy().reshape(-1, D).astype(np.float64)
        _assert_network_outputs(full[7][sl].cpu().numpy().reshape(-1), orc.value(last_rows, run=run), "bootstrap value", wd)
    assert bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all()) and full[3].shape == (T, TE, N)
    for e in (a, b, c):
        e.close()


@pytest.mark.parametrize("shape,E,T", [((4, 2, 3), 2048, 12), ((2, 1, 1), 200, 12), ((6, 2, 4), 512, 10), ((10, 3, 8), 100, 10)])
def test_teacher_forced_against_the_oracles_rollout(mods, shape, E, T):
    """The oracle runs free; before every step its state is forced into the library, which then does one
    actor-critic step: actions, log-probabilities, values and the bootstrap value against orc.rollout_ac."""
    say("tag actor-critic teacher-forced shape=%s E=%d" % (shape, E))
    env, orc = _env(mods, E, shape), _oracle(mods, E, shape)
    orc.reset(13)
    env.reset(13)
    bufs = env.empty_traj_ac(1)
    agree = total = 0
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
        Hp.assert_close_step(val, rval, "value")
        Hp.assert_close_step(logp[same], rlogp[same], "log-prob of the sampled action")
    say("  action agreement %.6f over %d" % (agree / total, total))
    assert (1.0 - agree / total) * total <= max(2, 1e-4 * total)
    env.close()


def test_errors_and_absent_outputs(mods):
    MpeEnv, _ = mods
    from paper_2311_10090_amd.binding import MpeError, MPE_EINVAL, MPE_ESTATE
    shape = (4, 2, 3)
    env = _env(mods, 200, shape, critic=False)
    env.reset(0)
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2)
    assert ei.value.code == MPE_ESTATE
    env.set_critic(*Hp.to_dev(_weights(shape, 1, 3)[1]))
    ref = _env(mods, 200, shape, critic=False)
    ref.reset(0)
    env.rollout_ac(7)                       # no outputs at all
    ref.rollout(7)
    for x, y in zip(env.get_state(), ref.get_state()):
        assert torch.equal(x, y) if hasattr(x, "shape") else x == y
    env.set_critic()                        # critic removed again
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2)
    assert ei.value.code == MPE_ESTATE
    env.close()
    ref.close()
    big = MpeEnv(Hp.tag_gpu_config(64, 6, 2, 4, 1, 128))              # networks of this scenario are 64 wide
    with pytest.raises(MpeError) as ei:
        big.set_critic(*Hp.to_dev(synth.critic_weights(0, 1, big.D, 128)))
    assert ei.value.code == MPE_EINVAL
    big.close()
    runs = _env(mods, 40, shape, R=2)                                  # several runs: multiples of 16 envs per run
    runs.reset(0)
    with pytest.raises(MpeError) as ei:
        runs.rollout_ac(2)
    assert ei.value.code == MPE_EINVAL
    runs.close()
