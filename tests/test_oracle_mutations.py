"""Do the oracle's pins notice a mistake?  Each entry below plants ONE plausible mistake (a dropped term, a
wrong sign or index, a swapped operand, a missing rounding point) in a COPY of oracle/mpe_oracle.cpp,
compiles the copy into a temporary folder and runs the pin tests against it; every mutant must make at
least one pin fail.  oracle/mpe_oracle.cpp itself is never touched, and nothing here runs on a GPU.

A survivor means that part of the oracle is pinned by nothing but its own formula."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mpe_oracle.cpp")

BASE = "tests/test_oracle_pins.py"
TAG = "tests/test_oracle_tag_pins.py"
GRU = "tests/test_oracle_gru_pins.py"

# (name, pin file, text in the source, replacement, which occurrence of the text)
MUTANTS = [
    # ---- Philox4x32-10 and the word conversions
    ("philox multiplier 0", BASE, "0xD2511F53u", "0xD2511F55u", 0),
    ("philox multiplier 1", BASE, "0xCD9E8D57u", "0xCD9E8D55u", 0),
    ("philox key increment 0", BASE, "k0 += 0x9E3779B9u;", "k0 += 0x9E3779B1u;", 0),
    ("philox key increment 1", BASE, "k1 += 0xBB67AE85u;", "k1 += 0xBB67AE83u;", 0),
    ("philox nine rounds", BASE, "round < 10", "round < 9", 0),
    ("philox crossed products", BASE, "const uint32_t n0 = hi1 ^ c1 ^ k0;", "const uint32_t n0 = hi0 ^ c1 ^ k0;", 0),
    ("philox key word reused", BASE, "const uint32_t n2 = hi0 ^ c3 ^ k1;", "const uint32_t n2 = hi0 ^ c3 ^ k0;", 0),
    ("position on a 23-bit grid", BASE, "double(w >> 8) * (1.0 / 8388608.0) - 1.0", "double(w >> 9) * (1.0 / 4194304.0) - 1.0", 0),
    ("uniform can be zero", BASE, "double(2u * (w >> 9) + 1u)", "double(2u * (w >> 9))", 0),
    ("uniform action by modulo", BASE, "int((uint64_t(w) * 5u) >> 32)", "int(w % 5u)", 0),
    # ---- reset
    ("reset counter fields swapped", BASE, "{uint32_t(o.cfg.env_offset + env), s, uint32_t(e), TAG_RESET_POS}",
     "{uint32_t(o.cfg.env_offset + env), uint32_t(e), s, TAG_RESET_POS}", 0),
    ("reset y from word 2", BASE, "double y = word_to_position(w[1]);", "double y = word_to_position(w[2]);", 0),
    ("reset key words swapped", BASE, "{o.seed, uint32_t(o.cfg.run_offset + run)}", "{uint32_t(o.cfg.run_offset + run), o.seed}", 0),
    ("reset keeps the velocity", BASE, "o.vel_a[(ge * o.N + e) * 2 + 0] = 0.0;", "", 0),
    ("reset keeps the episode counter", BASE, "  o.ep_step[ge] = 0;\n}", "}", 0),
    # ---- observation (simple spread: second occurrence of the shared lines)
    ("obs landmark sign", BASE, "ob[c++] = pl[2 * k + 0] - pa[2 * i + 0];", "ob[c++] = pa[2 * i + 0] - pl[2 * k + 0];", 1),
    ("obs other-agent sign", BASE, "ob[c++] = pa[2 * j + 1] - pa[2 * i + 1];", "ob[c++] = pa[2 * i + 1] - pa[2 * j + 1];", 1),
    ("obs velocity y repeated x", BASE, "ob[c++] = va[2 * i + 1];", "ob[c++] = va[2 * i + 0];", 1),
    ("obs comm slots not zero", BASE, "for (int z = 0; z < 2 * (o.N - 1); ++z) ob[c++] = 0.0;", "for (int z = 0; z < 2 * (o.N - 1); ++z) ob[c++] = 1.0;", 0),
    ("obs self not skipped", BASE, "      if (j == i) continue;\n      ob[c++] = pa[2 * j + 0] - pa[2 * i + 0];",
     "      if (j == o.N - 1 - i) continue;\n      ob[c++] = pa[2 * j + 0] - pa[2 * i + 0];", 1),
    # ---- transition (simple spread)
    ("action 1 pushes +x", BASE, "case 1: ux = -1.0; break;", "case 1: ux = +1.0; break;", 1),
    ("action 3 pushes x", BASE, "case 3: uy = -1.0; break;", "case 3: ux = -1.0; break;", 1),
    ("control force x from uy", BASE, "F[2 * i + 0] = c.accel * ux;", "F[2 * i + 0] = c.accel * uy;", 0),
    ("contact distance r instead of 2r", BASE, "softplus((2.0 * c.agent_radius - d) / c.contact_margin)", "softplus((c.agent_radius - d) / c.contact_margin)", 0),
    ("contact reaction same sign", BASE, "F[2 * j + 0] -= scale * dx;", "F[2 * j + 0] += scale * dx;", 0),
    ("contact force not normalised", BASE, "const double scale = c.contact_force * pen / std::max(d, 1e-12);", "const double scale = c.contact_force * pen;", 1),
    ("hard contact instead of softplus", BASE, "return std::max(x, 0.0) + std::log1p(std::exp(-std::fabs(x)));", "return std::max(x, 0.0);", 0),
    ("penetration without the margin factor", BASE, "const double pen = c.contact_margin * softplus((2.0", "const double pen = softplus((2.0", 0),
    ("velocity before position", BASE,
     "      pa[2 * i + a] += va[2 * i + a] * c.dt;\n      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;",
     "      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;\n      pa[2 * i + a] += va[2 * i + a] * c.dt;", 1),
    ("force times mass", BASE, "(F[2 * i + a] / c.mass) * c.dt;", "(F[2 * i + a] * c.mass) * c.dt;", 1),
    ("damping factor itself", BASE, "va[2 * i + a] * (1.0 - c.damping) +", "va[2 * i + a] * c.damping +", 1),
    ("position moves backwards", BASE, "pa[2 * i + a] += va[2 * i + a] * c.dt;", "pa[2 * i + a] -= va[2 * i + a] * c.dt;", 1),
    ("force without dt", BASE, "(F[2 * i + a] / c.mass) * c.dt;", "(F[2 * i + a] / c.mass);", 1),
    ("reward sign", BASE, "    r -= best;", "    r += best;", 0),
    ("reward: min over landmarks per agent", BASE,
     "      const double dx = pa[2 * i + 0] - pl[2 * k + 0];\n      const double dy = pa[2 * i + 1] - pl[2 * k + 1];\n      best = std::min(",
     "      const double dx = pa[2 * k + 0] - pl[2 * i + 0];\n      const double dy = pa[2 * k + 1] - pl[2 * i + 1];\n      best = std::min(", 0),
    ("reward: max instead of min", BASE, "    double best = INFINITY;\n    for (int i = 0; i < o.N; ++i) {\n      const double dx = pa[2 * i + 0] - pl[2 * k + 0];\n      const double dy = pa[2 * i + 1] - pl[2 * k + 1];\n      best = std::min(",
     "    double best = 0.0;\n    for (int i = 0; i < o.N; ++i) {\n      const double dx = pa[2 * i + 0] - pl[2 * k + 0];\n      const double dy = pa[2 * i + 1] - pl[2 * k + 1];\n      best = std::max(", 0),
    ("overlap at equality", BASE, "< 2.0 * c.agent_radius) ++overlaps;", "<= 2.0 * c.agent_radius) ++overlaps;", 0),
    ("overlap threshold r", BASE, "< 2.0 * c.agent_radius) ++overlaps;", "< c.agent_radius) ++overlaps;", 0),
    ("mixing weights swapped", BASE, "(1.0 - c.local_ratio) * r - c.local_ratio * double(overlaps)", "c.local_ratio * r - (1.0 - c.local_ratio) * double(overlaps)", 0),
    ("overlaps rewarded", BASE, "(1.0 - c.local_ratio) * r - c.local_ratio * double(overlaps)", "(1.0 - c.local_ratio) * r + c.local_ratio * double(overlaps)", 0),
    ("done one step late", BASE, "const bool d = o.ep_step[ge] >= c.max_episode_steps;", "const bool d = o.ep_step[ge] > c.max_episode_steps;", 1),
    ("auto-reset keyed by the old step", BASE, "if (d) reset_env(o, run, env, s + 1);", "if (d) reset_env(o, run, env, s);", 1),
    # ---- policy, critic, sampling
    ("W1 transposed", BASE, "acc += x[k] * W1[size_t(k) * H + j];", "acc += x[k] * W1[size_t(j) * D + k];", 0),
    ("b1 outside tanh", BASE, "h1[j] = std::tanh(acc + b1[j]);", "h1[j] = std::tanh(acc) + b1[j];", 0),
    ("b2 dropped", BASE, "h2[j] = std::tanh(acc + b2[j]);", "h2[j] = std::tanh(acc);", 0),
    ("b3 dropped", BASE, "z[a] = acc + b3[a];", "z[a] = acc;", 0),
    ("W3 transposed", BASE, "acc += h2[k] * W3[size_t(k) * nout + a];", "acc += h2[k] * W3[size_t(a) * H + k];", 0),
    ("layer 2 reads the observation width", BASE, "acc += h1[k] * W2[size_t(k) * H + j];", "acc += h1[k] * W2[size_t(j) * H + k];", 0),
    ("bf16: h1 not rounded", BASE, "if (bf) for (int j = 0; j < H; ++j) h1[j] = round_to_bf16(h1[j]);", "", 0),
    ("bf16: h2 not rounded", BASE, "if (bf) for (int j = 0; j < H; ++j) h2[j] = round_to_bf16(h2[j]);", "", 0),
    ("bf16: observation not rounded", BASE, "x[k] = bf ? round_to_bf16(ob[k]) : ob[k];", "x[k] = ob[k];", 0),
    ("bf16 by truncation", BASE, "const double r = std::nearbyint(scaled);", "const double r = std::trunc(scaled);", 0),
    ("bf16 with 7 significant bits", BASE, "const double scaled = std::ldexp(m, 8);", "const double scaled = std::ldexp(m, 7) * 2.0 + 0.25;", 0),
    ("gumbel: single log", BASE, "const double g = -std::log(-std::log(u));", "const double g = -std::log(u);", 0),
    ("gumbel: fifth word from word 1", BASE, "{w0[0], w0[1], w0[2], w0[3], w1[0]}", "{w0[0], w0[1], w0[2], w0[3], w1[1]}", 0),
    ("gumbel: words 1 and 2 swapped", BASE, "{w0[0], w0[1], w0[2], w0[3], w1[0]}", "{w0[0], w0[2], w0[1], w0[3], w1[0]}", 0),
    ("gumbel subtracted", BASE, "const double v = z[k] + g;", "const double v = z[k] - g;", 0),
    ("ties to the highest index", BASE, "if (v > best_v) { best_v = v; best = k; }", "if (v >= best_v) { best_v = v; best = k; }", 0),
    ("gumbel counter fields swapped", BASE, "const uint32_t c0[4] = {env, s, agent, TAG_GUMBEL0};", "const uint32_t c0[4] = {env, agent, s, TAG_GUMBEL0};", 0),
    ("uniform action from the reset stream", BASE, "const uint32_t c[4] = {env, s, agent, TAG_UNIFORM_ACTION};", "const uint32_t c[4] = {env, s, agent, TAG_RESET_POS};", 0),
    ("log-sum-exp without the shift added back", BASE, "const double lse = m + std::log(sum);", "const double lse = std::log(sum);", 0),
    ("log-probability of action 0", BASE, "logp[i] = lp[act[i]];", "logp[i] = lp[0];", 1),   # (0 is the recurrent branch)
    ("critic reads the policy's weights", BASE, "mlp_forward(o, o.critic, 1, run, ob, &v);", "mlp_forward(o, o.pol, 1, run, ob, &v);", 0),
    ("value of agent 0's row for every agent", BASE, "o.gru.set ? gv[i] : critic_value(o, run, ob.data() + size_t(i) * o.D);",
     "o.gru.set ? gv[i] : critic_value(o, run, ob.data());", 0),
    # ---- rollout
    ("rollout: step not advanced", BASE, "const uint32_t s = o.abs_step + uint32_t(t);", "const uint32_t s = o.abs_step;", 0),
    ("rollout: stale last_obs", BASE, "if (last_obs) observe_env(o, ge, last_obs + ge * row);", "if (last_obs) std::memcpy(last_obs + ge * row, ob.data(), row * sizeof(double));", 0),
    ("rollout: absolute step not carried", BASE, "  o.abs_step += uint32_t(T);\n  return 0;\n}\n\n// Actor-critic rollout", "  return 0;\n}\n\n// Actor-critic rollout", 0),
    # ---- second scenario
    ("tag: radii of the roles swapped", TAG, "return i < A ? c.adv_radius : c.agent_radius;", "return i < A ? c.agent_radius : c.adv_radius;", 0),
    ("tag: gains swapped", TAG, "return i < A ? c.adv_accel : c.accel;", "return i < A ? c.accel : c.adv_accel;", 0),
    ("tag: speed limits swapped", TAG, "return i < A ? c.adv_max_speed : c.good_max_speed;", "return i < A ? c.good_max_speed : c.adv_max_speed;", 0),
    ("tag: no speed limit", TAG, "if (speed > limit(i)) {", "if (false) {", 0),
    ("tag: clip without normalising", TAG, "va[2 * i + 0] = va[2 * i + 0] / speed * limit(i);", "va[2 * i + 0] = va[2 * i + 0] * limit(i);", 0),
    ("tag: obstacle contact distance", TAG, "radius(i) + c.landmark_radius, fx, fy);", "c.landmark_radius, fx, fy);", 0),
    ("tag: obstacle pulls", TAG, "radius(i) + c.landmark_radius, fx, fy);\n      F[2 * i + 0] += fx;", "radius(i) + c.landmark_radius, fx, fy);\n      F[2 * i + 0] -= fx;", 0),
    ("tag: pair contact distance", TAG, "radius(i) + radius(j), fx, fy);", "radius(i), fx, fy);", 0),
    ("tag: pair reaction same sign", TAG, "      F[2 * j + 1] -= fy;", "      F[2 * j + 1] += fy;", 0),
    ("tag: touching at equality", TAG, "return std::sqrt(dx * dx + dy * dy) < radius(i) + radius(j);", "return std::sqrt(dx * dx + dy * dy) <= radius(i) + radius(j);", 0),
    ("tag: adversary reward 5 per catch", TAG, "reward[i] = 10.0 * double(caught);", "reward[i] = 5.0 * double(caught);", 0),
    ("tag: good agent pays for every catch", TAG, "reward[g] = -10.0 * double(hits)", "reward[g] = -10.0 * double(caught)", 0),
    ("tag: y boundary penalty dropped", TAG, " - tag_bound(std::fabs(pa[2 * g + 1]));", ";", 0),
    ("tag: boundary slope", TAG, "return (u - 0.9) * 10.0;", "return (u - 0.9) * 1.0;", 0),
    ("tag: boundary exponent", TAG, "std::exp(2.0 * u - 2.0)", "std::exp(u - 1.0)", 0),
    ("tag: boundary starts at 0.8", TAG, "if (u < 0.9) return 0.0;", "if (u < 0.8) return 0.0;", 0),
    ("tag: boundary cap", TAG, "std::min(std::exp(2.0 * u - 2.0), 10.0)", "std::min(std::exp(2.0 * u - 2.0), 100.0)", 0),
    ("tag: velocities of the adversaries observed", TAG, "    for (int j = A; j < o.N; ++j) {\n      if (j == i) continue;\n      ob[c++] = va[2 * j + 0];",
     "    for (int j = 0; j < A; ++j) {\n      if (j == i) continue;\n      ob[c++] = va[2 * j + 0];", 0),
    ("tag: obstacle product in double", TAG, "x = double(float(x) * 0.9f);", "x = x * 0.9;", 0),
    ("tag: agents drawn in the inner box too", TAG, "if (o.cfg.scenario == 1 && e >= o.N) {", "if (o.cfg.scenario == 1) {", 0),
    ("tag: velocity before position", TAG,
     "      pa[2 * i + a] += va[2 * i + a] * c.dt;\n      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;",
     "      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;\n      pa[2 * i + a] += va[2 * i + a] * c.dt;", 0),
    ("tag: done one step late", TAG, "const bool d = o.ep_step[ge] >= c.max_episode_steps;", "const bool d = o.ep_step[ge] > c.max_episode_steps;", 0),
    ("tag: auto-reset keyed by the old step", TAG, "if (d) reset_env(o, run, env, s + 1);", "if (d) reset_env(o, run, env, s);", 0),
    ("tag: obs landmark sign", TAG, "ob[c++] = pl[2 * k + 1] - pa[2 * i + 1];", "ob[c++] = pa[2 * i + 1] - pl[2 * k + 1];", 0),
    # ---- recurrent policy
    ("gru: reset gate from the update columns", GRU, "const double r = sigmoid(gi[j] + gh[j]);", "const double r = sigmoid(gi[G + j] + gh[G + j]);", 0),
    ("gru: reset gate multiplies both products", GRU, "std::tanh(gi[2 * G + j] + r * gh[2 * G + j]);", "std::tanh(r * (gi[2 * G + j] + gh[2 * G + j]));", 0),
    ("gru: update gate inverted", GRU, "hn[j] = (1.0 - zz) * n + zz * h[j];", "hn[j] = zz * n + (1.0 - zz) * h[j];", 0),
    ("gru: carried state not rounded", GRU, "for (int k = 0; k < G; ++k) hb[k] = rnd(h[k]);", "for (int k = 0; k < G; ++k) hb[k] = h[k];", 0),
    ("gru: embedding not rounded", GRU, "e[j] = rnd(std::tanh(acc + be[j]));", "e[j] = std::tanh(acc + be[j]);", 0),
    ("gru: second layer without tanh", GRU, "y[j] = rnd(std::tanh(acc + bff[j]));", "y[j] = rnd(acc + bff[j]);", 0),
    ("gru: recurrent bias dropped", GRU, "gh[j] = ah + bh[j];", "gh[j] = ah;", 0),
    ("gru: state not carried", GRU, "  for (int j = 0; j < G; ++j) h[j] = hn[j];\n", "", 0),
    ("gru: Wi transposed", GRU, "ai += e[k] * Wi[size_t(k) * 3 * G + j];", "ai += e[k] * Wi[size_t(j) * G + k];", 0),
    ("gru: sigmoid of -x", GRU, "return 1.0 / (1.0 + std::exp(-x));", "return 1.0 / (1.0 + std::exp(x));", 0),
    ("gru: state survives an episode end", GRU, "if (d && o.gru.set) std::fill_n(", "if (false && o.gru.set) std::fill_n(", 0),
    ("gru: new state rounded before it is carried", GRU, "  for (int j = 0; j < G; ++j) h[j] = hn[j];\n", "  for (int j = 0; j < G; ++j) h[j] = rnd(hn[j]);\n", 0),
    ("gru: logits from the unrounded second layer", GRU, "y[j] = rnd(std::tanh(acc + bff[j]));", "y[j] = std::tanh(acc + bff[j]);", 0),
    # critic head of the recurrent actor-critic
    ("gru critic: hidden bias dropped", GRU, "v += rnd(std::tanh(acc + bc[j])) * wv[j];", "v += rnd(std::tanh(acc)) * wv[j];", 0),
    ("gru critic: output bias dropped", GRU, "double v = C.bv[size_t(run)];", "double v = 0.0;", 0),
    ("gru critic: Wc transposed", GRU, "acc += hb[k] * Wc[size_t(k) * G + j];", "acc += hb[k] * Wc[size_t(j) * G + k];", 0),
    ("gru critic: second layer not rounded", GRU, "v += rnd(std::tanh(acc + bc[j])) * wv[j];", "v += std::tanh(acc + bc[j]) * wv[j];", 0),
    ("gru critic: state not rounded", GRU, "for (int k = 0; k < G; ++k) hb[k] = rnd(hnew[k]);", "for (int k = 0; k < G; ++k) hb[k] = hnew[k];", 0),
    ("gru critic: value of the state before the step", GRU,
     "  for (int j = 0; j < G; ++j) h[j] = hn[j];\n  if (value) *value = gru_value(o, run, hn.data());",
     "  if (value) *value = gru_value(o, run, h);\n  for (int j = 0; j < G; ++j) h[j] = hn[j];", 0),
    ("gru critic: bootstrap value advances the carried state", GRU,
     "gru_forward(o, run, ob.data() + size_t(i) * o.D, hcopy.data(), z, &last_value[ge * o.N + i]);",
     "gru_forward(o, run, ob.data() + size_t(i) * o.D, &o.hidden[(ge * o.N + i) * GRU_H], z, &last_value[ge * o.N + i]);", 0),
    ("gru critic: log-probability of action 0", GRU, "logp[i] = lp[act[i]];", "logp[i] = lp[0];", 0),
    ("gru critic: value of agent 0 for all", GRU, "o.gru.set ? gv[i] : critic_value(", "o.gru.set ? gv[0] : critic_value(", 0),
    ("gru critic: output weights not rounded in bf16 mode", GRU, "load(o.gru_critic.wv, wv, R * G, b16);", "load(o.gru_critic.wv, wv, R * G, false);", 0),
]


def _nth_replace(text, old, new, n):
    idx = -1
    for _ in range(n + 1):
        idx = text.index(old, idx + 1)
    return text[:idx] + new + text[idx + len(old):]


def _run_mutant(args):
    k, (name, pins, old, new, occ), orig, tmp = args
    assert orig.count(old) > occ, "mutant %r: its text occurs %d times in the oracle (needs > %d)" % (name, orig.count(old), occ)
    src = os.path.join(tmp, "mutant_%03d.cpp" % k)
    lib = os.path.join(tmp, "mutant_%03d.so" % k)
    with open(src, "w") as f:
        f.write(_nth_replace(orig, old, new, occ))
    cc = subprocess.run(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-w", "-o", lib, src],
                        capture_output=True, text=True)
    if cc.returncode != 0:
        return name, "does not compile: " + cc.stderr[-300:]
    env = dict(os.environ, MPE_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", pins, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    os.remove(lib)
    if r.returncode == 1 and " failed" in r.stdout:
        return name, None                      # caught: a pin failed
    if r.returncode < 0:
        return name, None                      # caught: the mistake made the pins crash (out-of-range read or write)
    if r.returncode == 0:
        return name, "SURVIVED every pin of " + pins
    return name, "pins did not run (exit %d): %s" % (r.returncode, (r.stdout + r.stderr)[-300:])


def test_unmutated_copy_passes_through_the_same_route(tmp_path):
    """The route itself (copy, compile at -O1, load through MPE_ORACLE_LIB) keeps the pins green."""
    lib = str(tmp_path / "plain.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-w", "-o", lib, SRC])
    r = subprocess.run([sys.executable, "-m", "pytest", BASE, TAG, GRU, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=dict(os.environ, MPE_ORACLE_LIB=lib), capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("pins", [BASE, TAG, GRU])
def test_every_planted_mistake_is_caught(pins, tmp_path):
    orig = open(SRC).read()
    mine = [(k, m, orig, str(tmp_path)) for k, m in enumerate(MUTANTS) if m[1] == pins]
    assert len(mine) >= 10
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        results = list(ex.map(_run_mutant, mine))
    bad = ["%s: %s" % (name, why) for name, why in results if why]
    print("%d planted mistakes against %s, %d caught" % (len(results), pins, len(results) - len(bad)))
    assert not bad, "\n".join(bad)
