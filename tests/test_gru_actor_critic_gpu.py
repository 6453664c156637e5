"""Parity of the recurrent actor-critic rollout (mpe_set_gru_policy + mpe_set_gru_critic + mpe_rollout_ac)
against the oracle, through the C ABI.

Everything that is not the critic head's arithmetic is compared bit for bit: the rollout's plain outputs
and the carried state equal mpe_rollout's with the same recurrent policy, T steps equal T1 + T2 steps,
the bootstrap pass leaves the carried state alone.  The head's outputs (bf16 matrices and layer inputs,
fp32 sums) are held to the bar of the other bf16 networks: a value on a bf16 rounding boundary may round
the other way on the fp32 path and move an output by ~1e-3, so at least 90 % of the outputs meet the
single-step bar of 1e-5, all of them 2e-2, and the mean error stays below 1e-4."""
import numpy as np
import pytest
from scipy.special import log_softmax

from tests import helpers as Hp
from tests.test_gru_gpu import _bf16, _configs, say
from paper_2311_10090_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
G = 128


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.fail("gpu tests need a device; the library has no CPU fallback")
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    return MpeEnv, Oracle


def _env(mods, E, scn, R=1, wseed=3, head=True, max_ep=synth.MAX_EPISODE_STEPS, reward_mode=0):
    env = mods[0](_configs(E, scn, R, max_ep, reward_mode)[0])
    env.set_gru_policy(*Hp.to_dev(synth.gru_weights(wseed, R, env.D)))
    if head:
        env.set_gru_critic(*Hp.to_dev(synth.gru_critic_weights(wseed, R)))
    return env


def _oracle(mods, E, scn, R=1, wseed=3, max_ep=synth.MAX_EPISODE_STEPS):
    orc = mods[1](_configs(E, scn, R, max_ep)[1], threads=8)
    orc.set_gru(*synth.gru_weights(wseed, R, orc.D))
    orc.set_gru_critic(*synth.gru_critic_weights(wseed, R))
    return orc


def _assert_bf16_outputs(got, ref, what):
    err = np.abs(got - ref) / np.maximum(1.0, np.abs(ref))
    within = float((err <= Hp.STEP_RTOL).mean()) if err.size else 1.0
    say("  %s: %d outputs, within 1e-5 %.4f, mean %.2e, worst %.2e" % (what, err.size, within, err.mean() if err.size else 0.0,
                                                                      err.max(initial=0.0)))
    assert within >= 0.9 and err.max(initial=0.0) < 2e-2 and (err.size == 0 or err.mean() < 1e-4), what
    return within, float(err.max(initial=0.0))


SHAPES = [(8192, 3, 1), (200, 3, 1), (1, 3, 1), (129, 1, 1), (96, 2, 1), (64, 4, 1), (50, 6, 1), (40, 8, 1), (33, 10, 1),
          (64, 3, 3), (16, 5, 3), (32, 10, 2), (8192, (2, 1, 1), 1),
          (200, (4, 2, 3), 1), (100, (3, 0, 2), 1), (64, (6, 2, 4), 1), (70, (5, 2, 4), 1), (40, (8, 2, 6), 1), (33, (10, 3, 8), 1),
          (32, (4, 2, 3), 3), (16, (10, 3, 8), 2)]


@pytest.mark.parametrize("E,scn,R", SHAPES)
def test_plain_outputs_equal_mpe_rollout_and_steps_add_up(mods, E, scn, R):
    """The actor-critic rollout is mpe_rollout plus three outputs: the other five and the carried state are
    the same bits; T steps = T/2 + T/2 steps in every output (the carried state crosses the call and an
    episode end; the bootstrap pass of the first half must not have advanced it); absent outputs are not
    needed; and the head's outputs agree with the oracle's network on the recorded observations and
    carried states."""
    T = 30
    say("recurrent actor-critic E=%d scenario=%s R=%d" % (E, scn, R))
    a, b, c, d = _env(mods, E, scn, R), _env(mods, E, scn, R, head=False), _env(mods, E, scn, R), _env(mods, E, scn, R)
    N, D, TE = a.N, a.D, E * R
    for e in (a, b, c, d):
        e.reset(21)
    full = a.rollout_ac(T, *a.empty_traj_ac(T))
    plain = b.rollout(T, *b.empty_traj(T))
    for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
        assert torch.equal(full[k_ac], plain[k_pl]), "output %d differs from mpe_rollout" % k_ac
    assert torch.equal(a.get_hidden(), b.get_hidden())
    for x, y in zip(a.get_state(), b.get_state()):
        assert torch.equal(x, y) if hasattr(x, "shape") else x == y
    h1 = [x.clone() for x in c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))]
    assert bool(c.get_hidden().any())
    h2 = c.rollout_ac(T // 2, *c.empty_traj_ac(T // 2))
    for k in range(6):
        assert torch.equal(full[k], torch.cat([h1[k], h2[k]])), "continuation, output %d" % k
    assert torch.equal(full[6], h2[6]) and torch.equal(full[7], h2[7])
    assert torch.equal(a.get_hidden(), c.get_hidden())
    # without the bootstrap value (no extra pass) and without most outputs
    logp = torch.empty_like(full[2])
    val = torch.empty_like(full[3])
    d.rollout_ac(T, None, None, logp, val, None, None, None, None)
    assert torch.equal(logp, full[2]) and torch.equal(val, full[3]) and torch.equal(a.get_hidden(), d.get_hidden())
    assert bool((full[2] <= 0).all()) and bool(torch.isfinite(full[3]).all()) and full[3].shape == (T, TE, N)
    assert bool(full[5][24].all())
    # the network on the recorded inputs: one step at a time, the carried state read before every step
    orc = _oracle(mods, E, scn, R)
    c.reset(21)
    one = c.empty_traj_ac(1)
    steps = 8 if TE > 1000 else T
    got_lp, ref_lp, got_v, ref_v, got_lv, ref_lv = [], [], [], [], [], []
    for t in range(steps):
        h0 = c.get_hidden().cpu().numpy().astype(np.float64)
        obs, act, lp, v, rew, done, last, lastv = [x.cpu().numpy() for x in c.rollout_ac(1, *one)]
        assert np.array_equal(obs[0], full[0][t].cpu().numpy()) and np.array_equal(lp[0], full[2][t].cpu().numpy())
        assert np.array_equal(v[0], full[3][t].cpu().numpy())
        for run in range(R):
            sl = slice(run * E, (run + 1) * E)
            hn, z, rv = orc.gru_forward(obs[0, sl].reshape(-1, D), h0[sl].reshape(-1, G), run=run, with_value=True)
            ref_lp.append(log_softmax(z, axis=1)[np.arange(z.shape[0]), act[0, sl].reshape(-1)])
            got_lp.append(lp[0, sl].reshape(-1))
            ref_v.append(rv)
            got_v.append(v[0, sl].reshape(-1))
            # bootstrap value: the network once more on the observation after the step, from the state this
            # step left (zero where the episode ended)
            hn = np.where(np.repeat(done[0, sl], N)[:, None] != 0, 0.0, hn)
            _, _, rlv = orc.gru_forward(last[sl].reshape(-1, D), hn, run=run, with_value=True)
            ref_lv.append(rlv)
            got_lv.append(lastv[sl].reshape(-1))
    cat = np.concatenate
    w1 = _assert_bf16_outputs(cat(got_lp), cat(ref_lp), "log-prob from recorded obs, state and action")
    w2 = _assert_bf16_outputs(cat(got_v), cat(ref_v), "value from recorded obs and state")
    w3 = _assert_bf16_outputs(cat(got_lv), cat(ref_lv), "bootstrap value")
    Hp.record("recurrent actor-critic E=%d scenario=%s R=%d: log-prob / value / bootstrap value within 1e-5: %.4f / %.4f / %.4f, "
              "worst %.2e / %.2e / %.2e" % (E, scn, R, w1[0], w2[0], w3[0], w1[1], w2[1], w3[1]))
    for e in (a, b, c, d):
        e.close()


@pytest.mark.parametrize("E,scn,T", [(2048, 3, 12), (100, 1, 12), (130, 2, 12), (90, 5, 8), (64, 7, 6), (50, 10, 6),
                                     (512, (4, 2, 3), 10), (200, (2, 1, 1), 10), (64, (6, 2, 4), 8), (40, (10, 3, 8), 6)])
def test_teacher_forced_against_the_oracles_rollout(mods, E, scn, T):
    """The oracle runs free; before every step its state and carried state are forced into the library, which
    then does one actor-critic step: actions, log-probabilities, values, the bootstrap value and the new
    carried state against the oracle's own rollout_ac."""
    say("recurrent actor-critic teacher-forced E=%d scenario=%s" % (E, scn))
    env, orc = _env(mods, E, scn), _oracle(mods, E, scn)
    N = env.N
    orc.reset(13)
    env.reset(13)
    bufs = env.empty_traj_ac(1)
    agree = total = 0
    lp_g, lp_r, v_g, v_r, lv_g, lv_r = [], [], [], [], [], []
    rows_ok = 0
    for t in range(T):
        pa, va, pl, ep, s = orc.get_state()
        h0 = orc.get_hidden()
        env.set_state(*Hp.state_to_gpu(pa, va, pl, ep), 13, s)
        env.set_hidden(torch.from_numpy(h0.astype(np.float32)).cuda())
        robs, ract, rlogp, rval, rrew, rdone, rlast, rlastv = orc.rollout_ac(1)
        obs, act, logp, val, rew, done, last, lastv = [x.cpu().numpy() for x in env.rollout_ac(1, *bufs)]
        Hp.assert_close_step(obs, robs, "obs acted on")
        assert np.array_equal(done, rdone)
        same = act == ract
        agree += int(same.sum())
        total += same.size
        v_g.append(val.reshape(-1)); v_r.append(rval.reshape(-1))
        lp_g.append(logp[same]); lp_r.append(rlogp[same])
        # the observation after the step depends on every agent's action; and it reaches the network rounded to
        # bf16: where the two sides' observations (fp32 here, float64 there) round to different bf16 vectors,
        # which is common because contact-free velocities are exact ties of that rounding, the inputs differ
        # by a bf16 step and only the loose bound applies
        ok = same.all(axis=2)[0]
        same_input = (_bf16(last.astype(np.float64)) == _bf16(rlast)).all(axis=2) & ok[:, None]
        lv_g.append(lastv[same_input]); lv_r.append(rlastv[same_input])
        rows_ok += int(ok.sum()) * N
        loose = np.abs(lastv[ok] - rlastv[ok])
        assert loose.max(initial=0.0) < 2e-2
        h1, rh1 = env.get_hidden().cpu().numpy().astype(np.float64), orc.get_hidden()
        dh = np.abs(h1 - rh1)
        assert np.median(dh) < 1e-6 and dh.max() < 2e-2
        assert not h1[rdone[0] != 0].any()
    say("  action agreement %.6f over %d" % (agree / total, total))
    assert agree / total >= 0.9995
    cat = np.concatenate
    _assert_bf16_outputs(cat(v_g), cat(v_r), "value")
    _assert_bf16_outputs(cat(lp_g), cat(lp_r), "log-prob of the sampled action")
    _assert_bf16_outputs(cat(lv_g), cat(lv_r), "bootstrap value (rows whose observation rounds alike)")
    say("  rows whose next observation rounds alike on both sides: %d of %d" % (cat(lv_g).size, rows_ok))
    # (after the first step of an episode nearly every velocity is an exact tie, and a wide observation holds
    # many of them: the sample is a minority of the rows for the larger shapes; every row's bootstrap value is
    # checked from recorded inputs in the test above)
    assert cat(lv_g).size >= 200
    env.close()


@pytest.mark.parametrize("E,scn,R", [(256, 3, 1), (64, 3, 2), (48, 6, 1), (128, (4, 2, 3), 1)])
def test_free_running_episode_against_the_oracle(mods, E, scn, R):
    """A whole episode and its end, free running on both sides: on the envs whose sampled actions agree so
    far, values and log-probabilities follow the oracle's (the carried state feeds back, so earlier
    rounding flips are in them: the loose bar only, and the median tight)."""
    say("recurrent actor-critic free running E=%d scenario=%s R=%d" % (E, scn, R))
    env, orc = _env(mods, E, scn, R, wseed=9), _oracle(mods, E, scn, R, wseed=9)
    T = 27
    env.reset(7)
    orc.reset(7)
    obs, act, logp, val, rew, done, last, lastv = [x.cpu().numpy() for x in env.rollout_ac(T, *env.empty_traj_ac(T))]
    robs, ract, rlogp, rval, rrew, rdone, rlast, rlastv = orc.rollout_ac(T)
    assert np.array_equal(done, rdone) and bool(done[24].all())
    same = (act == ract).all(axis=2)
    alive = np.logical_and.accumulate(same, axis=0)
    say("  envs identical after 5 / 27 steps: %.3f / %.3f" % (alive[4].mean(), alive[-1].mean()))
    assert alive[4].mean() > 0.95 and alive[-1].mean() > 0.85
    prior = np.vstack([np.ones((1, E * R), bool), alive[:-1]])     # inputs of step t agree if the actions before it do
    for name, g, r, m in (("value", val, rval, prior), ("log-prob", logp, rlogp, alive), ("bootstrap value", lastv[None], rlastv[None], alive[-1:])):
        e = np.abs(g - r)[m]
        say("  %s: median %.2e, mean %.2e, worst %.2e over %d" % (name, np.median(e), e.mean(), e.max(), e.size))
        assert np.median(e) < 2e-6 and e.mean() < 5e-4 and e.max() < 5e-2, name
    env.close()


def test_head_management_and_refusals(mods):
    from paper_2311_10090_amd.binding import MpeError, MPE_EINVAL, MPE_ESTATE
    MpeEnv, _ = mods
    env = _env(mods, 64, 3, head=False)
    env.reset(5)
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2, *env.empty_traj_ac(2))
    assert ei.value.code == MPE_ESTATE and "mpe_set_gru_critic" in str(ei.value)
    head = Hp.to_dev(synth.gru_critic_weights(2, 1))
    with pytest.raises(MpeError) as ei:
        env.set_gru_critic(*head[:3], None)
    assert ei.value.code == MPE_EINVAL
    env.set_gru_critic(*head)
    v1 = env.rollout_ac(2, *env.empty_traj_ac(2))[3].clone()
    env.set_gru_critic(*Hp.to_dev(synth.gru_critic_weights(3, 1)))     # replaced: other values, same actions
    env.reset(5)
    v2 = env.rollout_ac(2, *env.empty_traj_ac(2))[3]
    assert not torch.equal(v1, v2)
    env.set_gru_critic()
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2, *env.empty_traj_ac(2))
    assert ei.value.code == MPE_ESTATE
    # the feed-forward critic is no substitute, and without the recurrent policy the head is not used
    env.set_gru_policy()
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2, *env.empty_traj_ac(2))
    assert ei.value.code == MPE_ESTATE
    env.close()
    for cfg in (Hp.gpu_config(64, 3, 1, 64, 0), Hp.gpu_config(64, 3, 1, 128, 0), Hp.tag_gpu_config(64, 4, 2, 3, 1, 64)):
        env = MpeEnv(cfg)
        with pytest.raises(MpeError) as ei:
            env.set_gru_critic(*head)
        assert ei.value.code == MPE_EINVAL
        env.close()
    # several runs whose size is not a multiple of 16
    env = _env(mods, 40, 3, R=2)
    env.reset(1)
    with pytest.raises(MpeError) as ei:
        env.rollout_ac(2, *env.empty_traj_ac(2))
    assert ei.value.code == MPE_EINVAL
    env.close()


def test_mixed_reward_and_short_episodes(mods):
    """The per-agent reward of simple spread and episodes that end every 4 steps (the carried state is cleared
    and the bootstrap pass starts from zero there): everything but the head's outputs equals mpe_rollout's."""
    E, T = 150, 17
    for kw in (dict(reward_mode=1), dict(max_ep=4)):
        a, b = _env(mods, E, 3, **kw), _env(mods, E, 3, head=False, **kw)
        a.reset(9)
        b.reset(9)
        full = a.rollout_ac(T, *a.empty_traj_ac(T))
        plain = b.rollout(T, *b.empty_traj(T))
        for k_ac, k_pl in ((0, 0), (1, 1), (4, 2), (5, 3), (6, 4)):
            assert torch.equal(full[k_ac], plain[k_pl]), "output %d differs from mpe_rollout (%s)" % (k_ac, kw)
        assert torch.equal(a.get_hidden(), b.get_hidden())
        if "max_ep" in kw:
            # T = 17: step 16 ended an episode?  no: episodes end at steps 3, 7, 11, 15; one step into the fifth
            assert bool(full[5][3].all()) and bool(full[5][15].all()) and not bool(full[5][16].any())
            orc = _oracle(mods, E, 3, max_ep=4)
            orc.reset(9)
            ref = orc.rollout_ac(T)
            same = (full[1].cpu().numpy() == ref[1]).all(axis=2)
            alive = np.logical_and.accumulate(same[12:], axis=0)[-1]     # the last episodes (reset states agree bit for bit)
            assert alive.mean() > 0.9
            e = np.abs(full[7].cpu().numpy() - ref[7])[alive]
            assert np.median(e) < 2e-6 and e.max() < 5e-2
            # a rollout that ends exactly at an episode end: the bootstrap value is that of a fresh episode
            a.reset(9)
            orc.reset(9)
            lv = a.rollout_ac(4, *a.empty_traj_ac(4))[7].cpu().numpy()
            rlv = orc.rollout_ac(4)[7]
            assert not a.get_hidden().any()
            e = np.abs(lv - rlv)
            assert np.median(e) < 2e-6 and e.max() < 2e-2
        a.close()
        b.close()
