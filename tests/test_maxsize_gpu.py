"""Very large batches: tens of millions of envs for a few steps, so that element indices and byte
offsets of the trajectory (and of the recurrent state) pass 2^32.  Env ranges at the start, at the
places where an index crosses 2^32, and at the (ragged) end are compared with the oracle, which
simulates envs [offset, offset + n) of the big job; the first steps after a reset leave no time
for rounding to grow, so everything is held to the episode bar and integer outputs are exact."""
import numpy as np
import pytest

from tests import helpers as Hp
from paper_2311_10090_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

T = 3


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.fail("gpu tests need a device; the library has no CPU fallback")
    from paper_2311_10090_amd.binding import MpeEnv
    from oracle import Oracle
    return MpeEnv, Oracle


def _ranges(E, row_floats, n=64):
    """First envs, last envs, and the envs around every place where the float index or the byte
    offset of an observation row passes a multiple of 2^32 inside the [T][E] trajectory."""
    out = {0, E - n}
    for t in range(T):
        for unit in (1, 4):   # floats, bytes
            lo, hi = t * E * row_floats * unit, (t + 1) * E * row_floats * unit
            k = lo // 2**32 + 1
            while k * 2**32 < hi:
                e = (k * 2**32 - lo) // (row_floats * unit)
                out.add(max(0, min(E - n, e - n // 2)))
                k += 1
    return sorted(out)


def _compare(outs, ref, off, n, what, exact_actions, min_agree=1.0):
    obs, act, rew, done, last = [x[:, off:off + n].cpu().numpy() if i < 4 else x[off:off + n].cpu().numpy()
                                 for i, x in enumerate(outs)]
    robs, ract, rrew, rdone, rlast = ref
    assert np.array_equal(done, rdone), what
    same = (act == ract).all(axis=2)
    alive = np.logical_and.accumulate(same, axis=0)
    if exact_actions:
        assert alive.all(), what
    else:
        assert alive[-1].mean() >= min_agree, what
    prior = np.vstack([np.ones((1, n), bool), alive[:-1]])
    e = np.abs(obs.astype(np.float64) - robs).reshape(T, n, -1).max(axis=2)
    assert (e * prior).max() <= Hp.EPISODE_ATOL, what
    el = np.abs(last.astype(np.float64) - rlast).reshape(n, -1).max(axis=1)
    assert (el * alive[-1]).max() <= Hp.EPISODE_ATOL, what
    r = np.abs(rew - rrew)
    r = r.max(axis=2) if r.ndim == 3 else r
    assert (r * alive).max() <= 1e-3, what
    return alive[-1]


@pytest.mark.parametrize("E,H", [(40_000_064, 0), (40_000_037, 0), (40_000_037, 64)])
def test_simple_spread_beyond_2_to_32(mods, E, H):
    """40 million envs x 3 steps: 6.5e9 observation floats.  Whole blocks (the wave-specialised
    env-only kernel), a ragged and misaligned size (the general kernel), and the fused fp32 kernel."""
    MpeEnv, Oracle = mods
    N = 3
    say("spread, %d envs, hidden %d" % (E, H))
    env = MpeEnv(Hp.gpu_config(E, N, 1, H, 0))
    w = synth.policy_weights_with_bias(4, 1, 6 * N, H) if H else None
    if w:
        env.set_policy(*Hp.to_dev(w))
    env.reset(3)
    outs = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    assert bool((outs[3] == 0).all()) and bool((outs[1] <= 4).all())
    for off in _ranges(E, N * 6 * N):
        orc = Oracle(Hp.oracle_config(64, N, 1, H, 0, env_offset=off), threads=4)
        if w:
            orc.set_policy(*w)
        orc.reset(3)
        _compare(outs, orc.rollout(T), off, 64, "envs %d.." % off, exact_actions=True)
    env.close()
    del outs
    torch.cuda.empty_cache()


def test_predator_prey_beyond_2_to_32(mods):
    MpeEnv, Oracle = mods
    E, shape = 30_000_001, (4, 2, 3)
    N = shape[0]
    say("tag, %d envs" % E)
    env = MpeEnv(Hp.tag_gpu_config(E, *shape, 1, 0))
    env.reset(5)
    outs = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    for off in _ranges(E, N * env.D):
        orc = Oracle(Hp.tag_oracle_config(64, *shape, 1, 0, env_offset=off), threads=4)
        orc.reset(5)
        _compare(outs, orc.rollout(T), off, 64, "envs %d.." % off, exact_actions=True)
    env.close()
    del outs
    torch.cuda.empty_cache()


def test_wide_bf16_beyond_2_to_32(mods):
    """4 million envs x 10 agents: 7.2e9 observation floats through the wide fused kernel."""
    MpeEnv, Oracle = mods
    E, N, H = 4_000_003, 10, 128
    say("wide bf16, %d envs" % E)
    env = MpeEnv(Hp.gpu_config(E, N, 1, H, 1))
    w = synth.policy_weights_with_bias(6, 1, 6 * N, H)
    env.set_policy(*Hp.to_dev(w))
    env.reset(7)
    outs = env.rollout(T, *env.empty_traj(T))
    torch.cuda.synchronize()
    ok = []
    for off in _ranges(E, N * 6 * N, n=32):
        orc = Oracle(Hp.oracle_config(32, N, 1, H, 1, env_offset=off), threads=4)
        orc.set_policy(*w)
        orc.reset(7)
        ok.append(_compare(outs, orc.rollout(T), off, 32, "envs %d.." % off, exact_actions=False, min_agree=0.9))
    assert np.concatenate(ok).mean() >= 0.97   # bf16 rounding flips may cost a few samples
    env.close()
    del outs
    torch.cuda.empty_cache()


def test_recurrent_state_beyond_2_to_32(mods):
    """12 million envs x 3 agents x 128 carried values: 4.6e9 floats of recurrent state."""
    MpeEnv, Oracle = mods
    E, N = 12_000_000, 3
    say("recurrent, %d envs" % E)
    env = MpeEnv(Hp.gpu_config(E, N, 1, 128, 1))
    w = synth.gru_weights(8, 1, 6 * N)
    env.set_gru_policy(*Hp.to_dev(w))
    env.reset(9)
    outs = env.rollout(T, *env.empty_traj(T))
    hid = env.get_hidden()
    torch.cuda.synchronize()
    offs = _ranges(E, N * 6 * N) + [2**32 // (N * 128) - 32, 2**32 // (4 * N * 128) - 32]   # state index, state byte offset
    for off in sorted(set(offs)):
        orc = Oracle(Hp.oracle_config(64, N, 1, 128, 1, env_offset=off), threads=4)
        orc.set_gru(*w)
        orc.reset(9)
        ok = _compare(outs, orc.rollout(T), off, 64, "envs %d.." % off, exact_actions=False, min_agree=0.9)
        d = np.abs(hid[off:off + 64].cpu().numpy().astype(np.float64) - orc.get_hidden())[ok]
        assert d.size and np.median(d) < 2e-3 and d.max() < 5e-2, "carried state of envs %d.." % off
    env.close()
    del outs, hid
    torch.cuda.empty_cache()
