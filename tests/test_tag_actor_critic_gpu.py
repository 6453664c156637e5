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


def _env(mods, E, shape, R=1, wseed=3, critic=True):
    env = mods[0](Hp.tag_gpu_config(E, *shape, R, 64))
    pw, cw = _weights(shape, R, wseed)
    env.set_policy(*Hp.to_dev(pw))
    if critic:
        env.set_critic(*Hp.to_dev(cw))
    return env


def _oracle(mods, E, shape, R=1, wseed=3):
    orc = mods[1](Hp.tag_oracle_config(E, *shape, R, 64), threads=8)
    pw, cw = _weights(shape, R, wseed)
    orc.set_policy(*pw)
    orc.set_critic(*cw)
    return orc


@pytest.mark.parametrize("shape,E,R", [((4, 2, 3), 1024, 1), ((4, 2, 3), 200, 1), ((4, 2, 3), 1, 1), ((4, 2, 3), 129, 1),
                                       ((2, 1, 1), 300, 1), ((2, 1, 1), 256, 1), ((3, 0, 2), 130, 1),
                                       ((4, 2, 3), 128, 3), ((2, 1, 1), 256, 2), ((3, 0, 2), 64, 2)])
def test_matches_plain_rollout_continues_and_agrees_with_the_oracles_networks(mods, shape, E, R):
    N, T = shape[0], 32
    D = Hp.tag_obs_dim(*shape)
    say("tag actor-critic shape=%s E=%d R=%d" % (shape, E, R))
    a, b, c = _env(mods, E, shape, R, 9), _env(mods, E, shape, R, 9, critic=False), _env(mods, E, shape, R, 9)
    orc = _oracle(mods, E, shape, R, 9)
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
        Hp.assert_close_step(logp[:, sl].reshape(-1), ref_lp, "log-prob from recorded obs and actions")
        Hp.assert_close_step(val[:, sl].reshape(-1), orc.value(rows, run=run), "value from recorded obs")
        last_rows = full[6][sl].cpu().numpy().reshape(-1, D).astype(np.float64)
        Hp.assert_close_step(full[7][sl].cpu().numpy().reshape(-1), orc.value(last_rows, run=run), "bootstrap value")
    assert bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all()) and full[3].shape == (T, TE, N)
    for e in (a, b, c):
        e.close()


@pytest.mark.parametrize("shape,E,T", [((4, 2, 3), 2048, 12), ((2, 1, 1), 200, 12)])
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
    bf = MpeEnv(Hp.tag_gpu_config(64, *shape, 1, 64, wd=1))          # bf16 weights: no actor-critic variant
    with pytest.raises(MpeError) as ei:
        bf.set_critic(*Hp.to_dev(_weights(shape, 1, 3)[1]))
    assert ei.value.code == MPE_EINVAL
    bf.close()
    big = MpeEnv(Hp.tag_gpu_config(64, 6, 2, 4, 1, 64))               # rows of 20 floats: no policy kernel
    with pytest.raises(MpeError) as ei:
        big.set_critic(*Hp.to_dev(synth.critic_weights(0, 1, 20, 64)))
    assert ei.value.code == MPE_EINVAL
    big.close()
    runs = _env(mods, 40, shape, R=2)                                  # several runs: multiples of 16 envs per run
    runs.reset(0)
    with pytest.raises(MpeError) as ei:
        runs.rollout_ac(2)
    assert ei.value.code == MPE_EINVAL
    runs.close()
