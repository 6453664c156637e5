// CPU oracle for the batched MPE simple-spread rollout (TEST INFRASTRUCTURE ONLY).
//
// This file is the plain, slow, scalar definition that the HIP library is checked
// against.  It is not part of the product: only the tests, the smoke check and the
// cpu_baseline leg of the benchmark may load it.  It shares no code, header, table
// or constant generator with the HIP path.
//
// What it follows.  The paper (JaxMARL, arXiv 2311.10090) describes MPE only as a 2-D
// world with simple physics in which particle agents move and interact with fixed
// landmarks (Sec. 3.1 "MPE", App. B.7), exposes it through reset(key) -> (obs, state)
// and step(key, state, actions) -> (obs, state, reward, done) with an explicit state
// and an explicit random key (App. C, API listing), uses a shared-parameter
// feed-forward policy with two tanh layers of width 64 for MPE (Sec. 3.2 "PPO";
// App. G, IPPO hyper-parameter table), and rolls out 128 steps per update (same
// table).  Everything quantitative the paper leaves open is fixed by the readings
// R-1 ... R-15 listed beside each function below.  R-14 is a second scenario (predator-prey,
// "simple tag") of the MPE family the paper says it implements in full (App. B.7); R-15 is the
// recurrent policy of the paper's headline speed figure (Fig. 3 caption; App. G, "Recurrent network").
//
// Arithmetic: double throughout (floating-point inputs arrive as float32 or double and
// are widened once).  No blocking, fusion or reordering: one loop per env, per step,
// per agent, in the order the definition states.
//
// Every function here is pinned by tests that do not depend on this file's own
// arithmetic: Philox known-answer vectors, hand-worked transitions, closed forms for
// a collision-free agent, contact-force magnitudes, invariants (antisymmetric
// contacts, momentum decay, permutation/translation/rotation invariance of the
// reward), brute-force re-derivations in numpy, a chi-square test of the sampler and
// a numpy float64 MLP chain.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------
// R-1  Random numbers: Philox4x32 with 10 rounds (Salmon et al., SC'11).
// Key = (seed, run).  Counter = (env index within the run, absolute step, entity or
// agent index, tag).
// ---------------------------------------------------------------------------------
enum : uint32_t { TAG_RESET_POS = 0, TAG_UNIFORM_ACTION = 1, TAG_GUMBEL0 = 2, TAG_GUMBEL1 = 3 };

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = uint64_t(0xD2511F53u) * uint64_t(c0);
    const uint64_t p1 = uint64_t(0xCD9E8D57u) * uint64_t(c2);
    const uint32_t hi0 = uint32_t(p0 >> 32), lo0 = uint32_t(p0);
    const uint32_t hi1 = uint32_t(p1 >> 32), lo1 = uint32_t(p1);
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Conversions of a 32-bit word (all exactly representable in float32).
//   position  in [-1, 1):  (w >> 8) * 2^-23 - 1
//   open-interval uniform in (0, 1): (2 * (w >> 9) + 1) * 2^-24
//   uniform action in {0..4}: floor(w * 5 / 2^32)
double word_to_position(uint32_t w) { return double(w >> 8) * (1.0 / 8388608.0) - 1.0; }
double word_to_open_uniform(uint32_t w) { return double(2u * (w >> 9) + 1u) * (1.0 / 16777216.0); }
int word_to_action(uint32_t w) { return int((uint64_t(w) * 5u) >> 32); }

struct Config {
  int32_t num_envs, num_agents, num_landmarks, num_runs, max_episode_steps;
  int32_t hidden, weight_dtype;  // weight_dtype: 0 = fp32 weights, 1 = bf16 weights + bf16 layer inputs
  int32_t env_offset, run_offset;  // this instance simulates envs [env_offset, env_offset+num_envs)
                                   // of runs [run_offset, run_offset+num_runs) of a larger job
  double dt, damping, mass, accel;
  double agent_radius, landmark_radius;
  double contact_force, contact_margin;
  int32_t reward_mode;   // 0: one shared coverage reward per env; 1: one mixed reward per agent (R-6b)
  int32_t reserved;
  double local_ratio;    // weight of the agent's own collision term in mode 1
  // scenario 1 (R-14, predator-prey): agents 0..num_adversaries-1 are adversaries, the rest are
  // good agents; agent_radius / accel above are the good agents' values
  int32_t scenario;        // 0: simple spread, 1: simple tag
  int32_t num_adversaries;
  double adv_radius, adv_accel, adv_max_speed, good_max_speed;
};

struct Policy {
  bool set = false;
  // Per run: W1[D][H], b1[H], W2[H][H], b2[H], W3[H][5], b3[5], row-major [fan_in][fan_out].
  std::vector<double> W1, b1, W2, b2, W3, b3;
};

// R-15 recurrent policy: per run We[D][G], be[G], Wi[G][3G], bi[3G], Wh[G][3G], bh[3G], Wf[G][G],
// bf[G], Wo[G][5], bo[5] with G = 128, row-major [fan_in][fan_out]; gate columns ordered r | z | n.
constexpr int GRU_H = 128;
struct GruPolicy {
  bool set = false;
  std::vector<double> We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo;
};

// R-16 critic head of the recurrent actor-critic: per run Wc[G][G], bc[G], wv[G], bv[1].
struct GruCritic {
  bool set = false;
  std::vector<double> Wc, bc, wv, bv;
};

struct Oracle {
  Config cfg;
  int E, N, L, R, D, H;
  uint32_t seed = 0;
  uint32_t abs_step = 0;
  bool was_reset = false;
  // State, plain array-of-structs: [run][env][entity][2].
  std::vector<double> pos_a, vel_a, pos_l;
  std::vector<int32_t> ep_step;
  Policy pol;
  Policy critic;   // same shape with ONE output: W3[H][1], b3[1]  (R-13)
  GruPolicy gru;                 // R-15; takes precedence over `pol` when set
  GruCritic gru_critic;          // R-16; used by the actor-critic rollout while `gru` is set
  std::vector<double> hidden;    // [run][env][agent][GRU_H], carried between steps and calls
  int nthreads = 1;
};

constexpr int NUM_ACTIONS = 5;

// Round a double to the nearest bfloat16 value (ties to even), returned as double.
// bfloat16 = sign, 8 exponent bits, 7 stored mantissa bits (the top half of float32).
// Values used here are far from the overflow/underflow limits of the format.
double round_to_bf16(double x) {
  if (x == 0.0 || !std::isfinite(x)) return x;
  int e;
  const double m = std::frexp(x, &e);              // x = m * 2^e, 0.5 <= |m| < 1
  const double scaled = std::ldexp(m, 8);          // 8 significant bits: 128 <= |scaled| < 256
  const double r = std::nearbyint(scaled);         // default rounding mode: ties to even
  return std::ldexp(r, e - 8);
}

// ---------------------------------------------------------------------------------
// R-2  Reset at absolute step s: every entity e (agents 0..N-1, then landmarks
// N..N+L-1) draws Philox(env, s, e, RESET_POS); words 0 and 1 give x and y on the
// 24-bit grid of [-1, 1).  Agent velocities are 0 and the episode counter is 0.
// Scenario 1 (R-14): landmark coordinates lie in [-0.9, 0.9): the grid value times 0.9, the
// product DEFINED as the float32 product of the two float32 numbers (so that the initial state
// is one exact float32 value on every implementation).
// ---------------------------------------------------------------------------------
void reset_env(Oracle& o, int run, int env, uint32_t s) {
  const uint32_t key[2] = {o.seed, uint32_t(o.cfg.run_offset + run)};
  const size_t ge = size_t(run) * o.E + env;
  for (int e = 0; e < o.N + o.L; ++e) {
    const uint32_t ctr[4] = {uint32_t(o.cfg.env_offset + env), s, uint32_t(e), TAG_RESET_POS};
    uint32_t w[4];
    philox4x32_10(ctr, key, w);
    double x = word_to_position(w[0]);
    double y = word_to_position(w[1]);
    if (o.cfg.scenario == 1 && e >= o.N) {
      x = double(float(x) * 0.9f);
      y = double(float(y) * 0.9f);
    }
    if (e < o.N) {
      o.pos_a[(ge * o.N + e) * 2 + 0] = x;
      o.pos_a[(ge * o.N + e) * 2 + 1] = y;
      o.vel_a[(ge * o.N + e) * 2 + 0] = 0.0;
      o.vel_a[(ge * o.N + e) * 2 + 1] = 0.0;
    } else {
      o.pos_l[(ge * o.L + (e - o.N)) * 2 + 0] = x;
      o.pos_l[(ge * o.L + (e - o.N)) * 2 + 1] = y;
    }
  }
  o.ep_step[ge] = 0;
}

// ---------------------------------------------------------------------------------
// R-8  Observation of agent i, length D = 4 + 2L + 4(N-1):
//   [ v_i, p_i, (l_k - p_i) for k ascending, (p_j - p_i) for j != i ascending,
//     2(N-1) zeros (the silent communication slots of the other agents) ].
// ---------------------------------------------------------------------------------
// R-14 observation (scenario 1), length D = 4 + 2L + 2(N-1) + 2G with G good agents:
//   [ v_i, p_i, (l_k - p_i) for k ascending, (p_j - p_i) for j != i ascending,
//     v_j for the good agents j != i ascending ].
// An adversary sees G velocities, a good agent G - 1: its row ends with two zeros so that every
// row has the same length (the shared network needs one input width).
void observe_env_tag(const Oracle& o, size_t ge, double* obs /* [N][D] */) {
  const double* pa = &o.pos_a[ge * o.N * 2];
  const double* va = &o.vel_a[ge * o.N * 2];
  const double* pl = o.pos_l.data() + ge * o.L * 2;   // (pos_l is empty without landmarks)
  const int A = o.cfg.num_adversaries;
  for (int i = 0; i < o.N; ++i) {
    double* ob = obs + size_t(i) * o.D;
    int c = 0;
    ob[c++] = va[2 * i + 0];
    ob[c++] = va[2 * i + 1];
    ob[c++] = pa[2 * i + 0];
    ob[c++] = pa[2 * i + 1];
    for (int k = 0; k < o.L; ++k) {
      ob[c++] = pl[2 * k + 0] - pa[2 * i + 0];
      ob[c++] = pl[2 * k + 1] - pa[2 * i + 1];
    }
    for (int j = 0; j < o.N; ++j) {
      if (j == i) continue;
      ob[c++] = pa[2 * j + 0] - pa[2 * i + 0];
      ob[c++] = pa[2 * j + 1] - pa[2 * i + 1];
    }
    for (int j = A; j < o.N; ++j) {
      if (j == i) continue;
      ob[c++] = va[2 * j + 0];
      ob[c++] = va[2 * j + 1];
    }
    while (c < o.D) ob[c++] = 0.0;
  }
}

void observe_env(const Oracle& o, size_t ge, double* obs /* [N][D] */) {
  if (o.cfg.scenario == 1) { observe_env_tag(o, ge, obs); return; }
  const double* pa = &o.pos_a[ge * o.N * 2];
  const double* va = &o.vel_a[ge * o.N * 2];
  const double* pl = o.pos_l.data() + ge * o.L * 2;   // (pos_l is empty without landmarks)
  for (int i = 0; i < o.N; ++i) {
    double* ob = obs + size_t(i) * o.D;
    int c = 0;
    ob[c++] = va[2 * i + 0];
    ob[c++] = va[2 * i + 1];
    ob[c++] = pa[2 * i + 0];
    ob[c++] = pa[2 * i + 1];
    for (int k = 0; k < o.L; ++k) {
      ob[c++] = pl[2 * k + 0] - pa[2 * i + 0];
      ob[c++] = pl[2 * k + 1] - pa[2 * i + 1];
    }
    for (int j = 0; j < o.N; ++j) {
      if (j == i) continue;
      ob[c++] = pa[2 * j + 0] - pa[2 * i + 0];
      ob[c++] = pa[2 * j + 1] - pa[2 * i + 1];
    }
    for (int z = 0; z < 2 * (o.N - 1); ++z) ob[c++] = 0.0;
  }
}

// softplus(x) = log(1 + exp(x)) in the overflow-safe form max(x,0) + log1p(exp(-|x|)).
double softplus(double x) { return std::max(x, 0.0) + std::log1p(std::exp(-std::fabs(x))); }

// ---------------------------------------------------------------------------------
// One transition of one env under given actions (readings R-3 ... R-7):
//  R-3 control force  F_i = accel * dir(a_i), dir: 0 none, 1 -x, 2 +x, 3 -y, 4 +y
//  R-4 contact force for every unordered agent pair (i, j) on the pre-step positions:
//        delta = p_i - p_j, d = |delta|, pen = margin * softplus((2 r - d) / margin),
//        f = contact_force * pen * delta / max(d, 1e-12);  F_i += f, F_j -= f.
//      Landmarks neither collide nor move.
//  R-5 integration: p_i += v_i * dt with the old velocity, then
//        v_i = v_i * (1 - damping) + (F_i / mass) * dt.   No speed clip.
//  R-6 reward on the post-step positions: r = - sum_k min_i |p_i - l_k|, one per env.
//  R-6b (reward_mode 1; the reward of the CPU lineage the paper's MPE port corresponds to, App. C
//      "environments correspond to existing CPU-based implementations"): agent i also pays 1 for
//      every other agent it overlaps after the step, c_i = #{ j != i : |p_i - p_j| < 2 r }, and
//      its reward mixes the two terms:  r_i = (1 - local_ratio) * r - local_ratio * c_i.
//      `reward` then holds N values.
//  R-7 ep_step += 1; done = (ep_step >= max_episode_steps).  If done, the env is reset
//      with the counter's step field set to s + 1, so the new episode depends only on
//      (seed, run, env, s + 1).
// ---------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------
// R-14  Second scenario, predator-prey ("simple tag"; paper App. B.7: all scenarios of the MPE
// family are implemented and their transitions match the CPU implementation; the paper prints
// none of it, so this is the reading taken, after the published CPU lineage):
//  roles    agents 0..A-1 are adversaries (radius adv_radius, control gain adv_accel, speed limit
//           adv_max_speed), agents A..N-1 are good agents (agent_radius, accel, good_max_speed);
//           L landmarks of radius landmark_radius are fixed obstacles.
//  forces   F_i = gain_i * dir(a_i).  Every unordered agent pair and every (agent, landmark) pair
//           collides, on the pre-step positions, with the contact law of R-4 and
//           d_min = sum of the two radii; a landmark pushes the agent and does not move.
//  motion   p_i += v_i * dt with the old velocity; v_i = v_i (1 - damping) + (F_i / mass) dt;
//           then, if |v_i| > limit_i, v_i is scaled to length limit_i.
//  reward   on the post-step positions, one value per agent.  Two entities touch when their centre
//           distance is strictly below the sum of their radii.  Every adversary gets
//           10 * #{(good g, adversary a) touching}.  A good agent g gets
//           -10 * #{adversaries touching g} - bound(|x_g|) - bound(|y_g|), with
//           bound(u) = 0 for u < 0.9, 10 (u - 0.9) for 0.9 <= u < 1, min(exp(2u - 2), 10) above.
//  episode  counter, done and auto-reset as in R-7.
// ---------------------------------------------------------------------------------
double tag_bound(double u) {
  if (u < 0.9) return 0.0;
  if (u < 1.0) return (u - 0.9) * 10.0;
  return std::min(std::exp(2.0 * u - 2.0), 10.0);
}

void step_env_tag(Oracle& o, int run, int env, uint32_t s, const uint8_t* act /* [N] */,
                  double* reward /* [N] */, uint8_t* done) {
  const Config& c = o.cfg;
  const size_t ge = size_t(run) * o.E + env;
  double* pa = &o.pos_a[ge * o.N * 2];
  double* va = &o.vel_a[ge * o.N * 2];
  const double* pl = o.pos_l.data() + ge * o.L * 2;   // (pos_l is empty without landmarks)
  const int A = c.num_adversaries;
  auto radius = [&](int i) { return i < A ? c.adv_radius : c.agent_radius; };
  auto gain = [&](int i) { return i < A ? c.adv_accel : c.accel; };
  auto limit = [&](int i) { return i < A ? c.adv_max_speed : c.good_max_speed; };
  // contact force on the first entity of a pair with separation (dx, dy) and contact distance dmin
  auto contact = [&](double dx, double dy, double dmin, double& fx, double& fy) {
    const double d = std::sqrt(dx * dx + dy * dy);
    const double pen = c.contact_margin * softplus((dmin - d) / c.contact_margin);
    const double scale = c.contact_force * pen / std::max(d, 1e-12);
    fx = scale * dx;
    fy = scale * dy;
  };

  std::vector<double> F(size_t(o.N) * 2, 0.0);
  for (int i = 0; i < o.N; ++i) {
    double ux = 0.0, uy = 0.0;
    switch (act[i]) {
      case 1: ux = -1.0; break;
      case 2: ux = +1.0; break;
      case 3: uy = -1.0; break;
      case 4: uy = +1.0; break;
      default: break;
    }
    F[2 * i + 0] = gain(i) * ux;
    F[2 * i + 1] = gain(i) * uy;
  }
  for (int i = 0; i < o.N; ++i) {
    for (int j = i + 1; j < o.N; ++j) {
      double fx, fy;
      contact(pa[2 * i + 0] - pa[2 * j + 0], pa[2 * i + 1] - pa[2 * j + 1], radius(i) + radius(j), fx, fy);
      F[2 * i + 0] += fx;
      F[2 * i + 1] += fy;
      F[2 * j + 0] -= fx;
      F[2 * j + 1] -= fy;
    }
  }
  for (int i = 0; i < o.N; ++i) {
    for (int k = 0; k < o.L; ++k) {
      double fx, fy;
      contact(pa[2 * i + 0] - pl[2 * k + 0], pa[2 * i + 1] - pl[2 * k + 1], radius(i) + c.landmark_radius, fx, fy);
      F[2 * i + 0] += fx;
      F[2 * i + 1] += fy;
    }
  }
  for (int i = 0; i < o.N; ++i) {
    for (int a = 0; a < 2; ++a) {
      pa[2 * i + a] += va[2 * i + a] * c.dt;
      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;
    }
    const double speed = std::sqrt(va[2 * i] * va[2 * i] + va[2 * i + 1] * va[2 * i + 1]);
    if (speed > limit(i)) {
      va[2 * i + 0] = va[2 * i + 0] / speed * limit(i);
      va[2 * i + 1] = va[2 * i + 1] / speed * limit(i);
    }
  }
  auto touching = [&](int i, int j) {
    const double dx = pa[2 * i + 0] - pa[2 * j + 0];
    const double dy = pa[2 * i + 1] - pa[2 * j + 1];
    return std::sqrt(dx * dx + dy * dy) < radius(i) + radius(j);
  };
  int caught = 0;   // touching (good, adversary) pairs
  for (int g = A; g < o.N; ++g)
    for (int a = 0; a < A; ++a)
      if (touching(g, a)) ++caught;
  for (int i = 0; i < A; ++i) reward[i] = 10.0 * double(caught);
  for (int g = A; g < o.N; ++g) {
    int hits = 0;
    for (int a = 0; a < A; ++a)
      if (touching(g, a)) ++hits;
    reward[g] = -10.0 * double(hits) - tag_bound(std::fabs(pa[2 * g + 0])) - tag_bound(std::fabs(pa[2 * g + 1]));
  }
  o.ep_step[ge] += 1;
  const bool d = o.ep_step[ge] >= c.max_episode_steps;
  *done = d ? 1 : 0;
  if (d) reset_env(o, run, env, s + 1);
}

void step_env(Oracle& o, int run, int env, uint32_t s, const uint8_t* act /* [N] */,
              double* reward /* [1], or [N] in reward_mode 1 and in scenario 1 */, uint8_t* done) {
  if (o.cfg.scenario == 1) { step_env_tag(o, run, env, s, act, reward, done); return; }
  const Config& c = o.cfg;
  const size_t ge = size_t(run) * o.E + env;
  double* pa = &o.pos_a[ge * o.N * 2];
  double* va = &o.vel_a[ge * o.N * 2];
  const double* pl = o.pos_l.data() + ge * o.L * 2;   // (pos_l is empty without landmarks)

  std::vector<double> F(size_t(o.N) * 2, 0.0);
  for (int i = 0; i < o.N; ++i) {
    double ux = 0.0, uy = 0.0;
    switch (act[i]) {
      case 1: ux = -1.0; break;
      case 2: ux = +1.0; break;
      case 3: uy = -1.0; break;
      case 4: uy = +1.0; break;
      default: break;
    }
    F[2 * i + 0] = c.accel * ux;
    F[2 * i + 1] = c.accel * uy;
  }
  for (int i = 0; i < o.N; ++i) {
    for (int j = i + 1; j < o.N; ++j) {
      const double dx = pa[2 * i + 0] - pa[2 * j + 0];
      const double dy = pa[2 * i + 1] - pa[2 * j + 1];
      const double d = std::sqrt(dx * dx + dy * dy);
      const double pen = c.contact_margin * softplus((2.0 * c.agent_radius - d) / c.contact_margin);
      const double scale = c.contact_force * pen / std::max(d, 1e-12);
      F[2 * i + 0] += scale * dx;
      F[2 * i + 1] += scale * dy;
      F[2 * j + 0] -= scale * dx;
      F[2 * j + 1] -= scale * dy;
    }
  }
  for (int i = 0; i < o.N; ++i) {
    for (int a = 0; a < 2; ++a) {
      pa[2 * i + a] += va[2 * i + a] * c.dt;
      va[2 * i + a] = va[2 * i + a] * (1.0 - c.damping) + (F[2 * i + a] / c.mass) * c.dt;
    }
  }
  double r = 0.0;
  for (int k = 0; k < o.L; ++k) {
    double best = INFINITY;
    for (int i = 0; i < o.N; ++i) {
      const double dx = pa[2 * i + 0] - pl[2 * k + 0];
      const double dy = pa[2 * i + 1] - pl[2 * k + 1];
      best = std::min(best, std::sqrt(dx * dx + dy * dy));
    }
    r -= best;
  }
  if (c.reward_mode == 1) {
    for (int i = 0; i < o.N; ++i) {
      int overlaps = 0;
      for (int j = 0; j < o.N; ++j) {
        if (j == i) continue;
        const double dx = pa[2 * i + 0] - pa[2 * j + 0];
        const double dy = pa[2 * i + 1] - pa[2 * j + 1];
        if (std::sqrt(dx * dx + dy * dy) < 2.0 * c.agent_radius) ++overlaps;
      }
      reward[i] = (1.0 - c.local_ratio) * r - c.local_ratio * double(overlaps);
    }
  } else {
    *reward = r;
  }
  o.ep_step[ge] += 1;
  const bool d = o.ep_step[ge] >= c.max_episode_steps;
  *done = d ? 1 : 0;
  if (d) reset_env(o, run, env, s + 1);
}

// ---------------------------------------------------------------------------------
// R-9  Policy: h1 = tanh(W1^T o + b1); h2 = tanh(W2^T h1 + b2); z = W3^T h2 + b3, with
// W stored row-major [fan_in][fan_out] (paper: two hidden layers, tanh, parameters
// shared by all agents).  bf16 mode: weights were rounded to bf16 when set; o, h1 and
// h2 are rounded to bf16 where they enter a layer; products, sums, biases and tanh stay
// in the wide type.
// ---------------------------------------------------------------------------------
void mlp_forward(const Oracle& o, const Policy& P, int nout, int run, const double* ob, double* z /* [nout] */) {
  const int D = o.D, H = o.H;
  const bool bf = o.cfg.weight_dtype == 1;
  const double* W1 = &P.W1[size_t(run) * D * H];
  const double* b1 = &P.b1[size_t(run) * H];
  const double* W2 = &P.W2[size_t(run) * H * H];
  const double* b2 = &P.b2[size_t(run) * H];
  const double* W3 = &P.W3[size_t(run) * H * nout];
  const double* b3 = &P.b3[size_t(run) * nout];
  std::vector<double> x(D), h1(H), h2(H);
  for (int k = 0; k < D; ++k) x[k] = bf ? round_to_bf16(ob[k]) : ob[k];
  for (int j = 0; j < H; ++j) {
    double acc = 0.0;
    for (int k = 0; k < D; ++k) acc += x[k] * W1[size_t(k) * H + j];
    h1[j] = std::tanh(acc + b1[j]);
  }
  if (bf) for (int j = 0; j < H; ++j) h1[j] = round_to_bf16(h1[j]);
  for (int j = 0; j < H; ++j) {
    double acc = 0.0;
    for (int k = 0; k < H; ++k) acc += h1[k] * W2[size_t(k) * H + j];
    h2[j] = std::tanh(acc + b2[j]);
  }
  if (bf) for (int j = 0; j < H; ++j) h2[j] = round_to_bf16(h2[j]);
  for (int a = 0; a < nout; ++a) {
    double acc = 0.0;
    for (int k = 0; k < H; ++k) acc += h2[k] * W3[size_t(k) * nout + a];
    z[a] = acc + b3[a];
  }
}

void policy_logits(const Oracle& o, int run, const double* ob, double* z /* [5] */) {
  mlp_forward(o, o.pol, NUM_ACTIONS, run, ob, z);
}

// ---------------------------------------------------------------------------------
// R-13  What an actor-critic learner (the paper's IPPO / MAPPO, Sec. 3.2; App. G: feed-forward
// networks of two tanh layers of width 64) takes from a rollout besides obs, action, reward and
// done: the log-probability of the sampled action under the categorical policy,
//     log pi(a | o) = z_a - ln sum_k exp(z_k),
// and the critic's value of the observation acted on.  The critic is a second network of the
// same shape with one output (the paper does not print the critic; this is the reading taken),
// fed the agent's own observation.
// ---------------------------------------------------------------------------------
void log_probs(const double* z, double* lp /* [5] */) {
  double m = z[0];
  for (int k = 1; k < NUM_ACTIONS; ++k) m = std::max(m, z[k]);
  double sum = 0.0;
  for (int k = 0; k < NUM_ACTIONS; ++k) sum += std::exp(z[k] - m);
  const double lse = m + std::log(sum);
  for (int k = 0; k < NUM_ACTIONS; ++k) lp[k] = z[k] - lse;
}

double critic_value(const Oracle& o, int run, const double* ob) {
  double v;
  mlp_forward(o, o.critic, 1, run, ob, &v);
  return v;
}

// ---------------------------------------------------------------------------------
// R-15  Recurrent policy (paper Fig. 3: an RNN agent on MPE; App. G "Recurrent network": hidden
// width 128, two fully-connected layers of width 128; activation tanh per the MPE column).  The
// paper prints no equations; the reading taken is the standard gated recurrent unit between the two
// fully-connected layers, parameters shared by all agents, one hidden vector h per agent:
//     e  = tanh(We^T o + be)                                 (first fully-connected layer)
//     r  = sigma(Wi_r^T e + bi_r + Wh_r^T h + bh_r)
//     z  = sigma(Wi_z^T e + bi_z + Wh_z^T h + bh_z)
//     n  = tanh (Wi_n^T e + bi_n + r * (Wh_n^T h + bh_n))
//     h' = (1 - z) * n + z * h
//     y  = tanh(Wf^T h' + bf)                                (second fully-connected layer)
//     logits = Wo^T y + bo
// h is zero at the start of an episode (after reset and after every done) and is carried across
// rollout calls.  bf16 mode (weight_dtype 1): the weight matrices were rounded to bf16 when set;
// o, e, h, h' and y are rounded to bf16 where they enter a matrix product; sums, biases, sigma, tanh,
// the gate arithmetic and the carried h stay in the wide type.
// ---------------------------------------------------------------------------------
double sigmoid(double x) { return 1.0 / (1.0 + std::exp(-x)); }

// R-16  Critic of the recurrent actor-critic.  The paper's PPO baselines are actor-critic (Sec. 3.2; App. G lists a
// value loss coefficient) and its recurrent network has two fully-connected layers of width 128 around the
// recurrent unit (App. G "Recurrent network"); the critic is not printed.  Reading taken: actor and critic
// share the first fully-connected layer and the recurrent unit, and the critic has a second fully-connected
// layer of its own and one output, fed the NEW carried state h' of the step:
//     yc = tanh(Wc^T h' + bc),   value = wv^T yc + bv
// with the rounding points of R-15 (h' and yc are rounded to bf16 where they enter a product).
double gru_value(const Oracle& o, int run, const double* hnew /* [GRU_H] */) {
  const int G = GRU_H;
  const GruCritic& C = o.gru_critic;
  const bool bf = o.cfg.weight_dtype == 1;
  auto rnd = [&](double v) { return bf ? round_to_bf16(v) : v; };
  const double* Wc = &C.Wc[size_t(run) * G * G];
  const double* bc = &C.bc[size_t(run) * G];
  const double* wv = &C.wv[size_t(run) * G];
  std::vector<double> hb(G);
  for (int k = 0; k < G; ++k) hb[k] = rnd(hnew[k]);
  double v = C.bv[size_t(run)];
  for (int j = 0; j < G; ++j) {
    double acc = 0.0;
    for (int k = 0; k < G; ++k) acc += hb[k] * Wc[size_t(k) * G + j];
    v += rnd(std::tanh(acc + bc[j])) * wv[j];
  }
  return v;
}

// `value` (nullable): the critic head of R-16 on the new carried state.
void gru_forward(const Oracle& o, int run, const double* ob, double* h /* [GRU_H] in/out */, double* z5 /* [5] */,
                 double* value = nullptr) {
  const int D = o.D, G = GRU_H;
  const GruPolicy& P = o.gru;
  const bool bf = o.cfg.weight_dtype == 1;
  auto rnd = [&](double v) { return bf ? round_to_bf16(v) : v; };
  const double* We = &P.We[size_t(run) * D * G];
  const double* be = &P.be[size_t(run) * G];
  const double* Wi = &P.Wi[size_t(run) * G * 3 * G];
  const double* bi = &P.bi[size_t(run) * 3 * G];
  const double* Wh = &P.Wh[size_t(run) * G * 3 * G];
  const double* bh = &P.bh[size_t(run) * 3 * G];
  const double* Wf = &P.Wf[size_t(run) * G * G];
  const double* bff = &P.bf[size_t(run) * G];
  const double* Wo = &P.Wo[size_t(run) * G * NUM_ACTIONS];
  const double* bo = &P.bo[size_t(run) * NUM_ACTIONS];
  std::vector<double> x(D), e(G), hb(G), gi(3 * G), gh(3 * G), hn(G), y(G);
  for (int k = 0; k < D; ++k) x[k] = rnd(ob[k]);
  for (int j = 0; j < G; ++j) {
    double acc = 0.0;
    for (int k = 0; k < D; ++k) acc += x[k] * We[size_t(k) * G + j];
    e[j] = rnd(std::tanh(acc + be[j]));
  }
  for (int k = 0; k < G; ++k) hb[k] = rnd(h[k]);
  for (int j = 0; j < 3 * G; ++j) {
    double ai = 0.0, ah = 0.0;
    for (int k = 0; k < G; ++k) {
      ai += e[k] * Wi[size_t(k) * 3 * G + j];
      ah += hb[k] * Wh[size_t(k) * 3 * G + j];
    }
    gi[j] = ai + bi[j];
    gh[j] = ah + bh[j];
  }
  for (int j = 0; j < G; ++j) {
    const double r = sigmoid(gi[j] + gh[j]);
    const double zz = sigmoid(gi[G + j] + gh[G + j]);
    const double n = std::tanh(gi[2 * G + j] + r * gh[2 * G + j]);
    hn[j] = (1.0 - zz) * n + zz * h[j];
  }
  for (int j = 0; j < G; ++j) h[j] = hn[j];
  if (value) *value = gru_value(o, run, hn.data());
  for (int k = 0; k < G; ++k) hb[k] = rnd(hn[k]);
  for (int j = 0; j < G; ++j) {
    double acc = 0.0;
    for (int k = 0; k < G; ++k) acc += hb[k] * Wf[size_t(k) * G + j];
    y[j] = rnd(std::tanh(acc + bff[j]));
  }
  for (int a = 0; a < NUM_ACTIONS; ++a) {
    double acc = 0.0;
    for (int k = 0; k < G; ++k) acc += y[k] * Wo[size_t(k) * NUM_ACTIONS + a];
    z5[a] = acc + bo[a];
  }
}

// ---------------------------------------------------------------------------------
// R-10  Gumbel-max sampling: g_k = -ln(-ln u_k); u_0..u_3 are the four words of
// Philox(env, s, agent, GUMBEL0), u_4 is word 0 of Philox(env, s, agent, GUMBEL1);
// action = argmax_k (z_k + g_k), lowest index on ties.
// Without a policy the action is floor(5 * w / 2^32) with w = word 0 of
// Philox(env, s, agent, UNIFORM_ACTION).
// ---------------------------------------------------------------------------------
int gumbel_max_action(uint32_t seed, uint32_t run, uint32_t env, uint32_t s, uint32_t agent,
                      const double* z) {
  const uint32_t key[2] = {seed, run};
  const uint32_t c0[4] = {env, s, agent, TAG_GUMBEL0};
  const uint32_t c1[4] = {env, s, agent, TAG_GUMBEL1};
  uint32_t w0[4], w1[4];
  philox4x32_10(c0, key, w0);
  philox4x32_10(c1, key, w1);
  const uint32_t words[NUM_ACTIONS] = {w0[0], w0[1], w0[2], w0[3], w1[0]};
  int best = 0;
  double best_v = -INFINITY;
  for (int k = 0; k < NUM_ACTIONS; ++k) {
    const double u = word_to_open_uniform(words[k]);
    const double g = -std::log(-std::log(u));
    const double v = z[k] + g;
    if (v > best_v) { best_v = v; best = k; }
  }
  return best;
}

int uniform_action(uint32_t seed, uint32_t run, uint32_t env, uint32_t s, uint32_t agent) {
  const uint32_t key[2] = {seed, run};
  const uint32_t c[4] = {env, s, agent, TAG_UNIFORM_ACTION};
  uint32_t w[4];
  philox4x32_10(c, key, w);
  return word_to_action(w[0]);
}

void choose_actions(Oracle& o, int run, int env, uint32_t s, const double* obs /* [N][D] */,
                    uint8_t* act /* [N] */, double* logp = nullptr /* [N], needs a policy */,
                    double* gru_values = nullptr /* [N], recurrent actor-critic only */) {
  for (int i = 0; i < o.N; ++i) {
    if (o.gru.set) {
      double z[NUM_ACTIONS];
      double* h = &o.hidden[((size_t(run) * o.E + env) * o.N + i) * GRU_H];
      gru_forward(o, run, obs + size_t(i) * o.D, h, z, gru_values ? gru_values + i : nullptr);
      act[i] = uint8_t(gumbel_max_action(o.seed, uint32_t(o.cfg.run_offset + run),
                                         uint32_t(o.cfg.env_offset + env), s, uint32_t(i), z));
      if (logp) {
        double lp[NUM_ACTIONS];
        log_probs(z, lp);
        logp[i] = lp[act[i]];
      }
    } else if (o.pol.set) {
      double z[NUM_ACTIONS];
      policy_logits(o, run, obs + size_t(i) * o.D, z);
      act[i] = uint8_t(gumbel_max_action(o.seed, uint32_t(o.cfg.run_offset + run),
                                         uint32_t(o.cfg.env_offset + env), s, uint32_t(i), z));
      if (logp) {
        double lp[NUM_ACTIONS];
        log_probs(z, lp);
        logp[i] = lp[act[i]];
      }
    } else {
      act[i] = uint8_t(uniform_action(o.seed, uint32_t(o.cfg.run_offset + run),
                                      uint32_t(o.cfg.env_offset + env), s, uint32_t(i)));
    }
  }
}

// ---------------------------------------------------------------------------------
// R-11  Rollout of T steps: for t = 0..T-1 record the current observation, choose the
// actions (policy + Gumbel-max, or uniform), record them, apply one transition, record
// reward and done.  After the loop last_obs is the current observation.  Actor-critic outputs
// (R-13, all nullable): logp_traj, value_traj [T][TE][N] and last_value [TE][N], the value of
// last_obs.  With the recurrent policy (R-16) the value of step t is the critic head on the carried state
// that step t produces, and last_value is the value that one more network evaluation on last_obs would
// give; that evaluation does not advance the carried state.
// ---------------------------------------------------------------------------------
void rollout_range(Oracle& o, size_t g0, size_t g1, int T, double* obs_traj, uint8_t* act_traj,
                   double* rew_traj, uint8_t* done_traj, double* last_obs, double* logp_traj = nullptr,
                   double* value_traj = nullptr, double* last_value = nullptr) {
  const size_t TE = size_t(o.R) * o.E;
  const size_t row = size_t(o.N) * o.D;
  std::vector<double> ob(row);
  std::vector<uint8_t> act(o.N);
  const size_t RW = (o.cfg.reward_mode == 1 || o.cfg.scenario == 1) ? size_t(o.N) : 1;   // rewards per env and step
  std::vector<double> r(RW);
  for (size_t ge = g0; ge < g1; ++ge) {
    const int run = int(ge / o.E), env = int(ge % o.E);
    for (int t = 0; t < T; ++t) {
      const uint32_t s = o.abs_step + uint32_t(t);
      observe_env(o, ge, ob.data());
      if (obs_traj) std::memcpy(obs_traj + (size_t(t) * TE + ge) * row, ob.data(), row * sizeof(double));
      std::vector<double> lp(o.N), gv(o.N);
      const bool rec_value = o.gru.set && value_traj != nullptr;
      choose_actions(o, run, env, s, ob.data(), act.data(), logp_traj ? lp.data() : nullptr,
                     rec_value ? gv.data() : nullptr);
      if (act_traj) std::memcpy(act_traj + (size_t(t) * TE + ge) * o.N, act.data(), o.N);
      if (logp_traj) std::memcpy(logp_traj + (size_t(t) * TE + ge) * o.N, lp.data(), o.N * sizeof(double));
      if (value_traj)
        for (int i = 0; i < o.N; ++i)
          value_traj[(size_t(t) * TE + ge) * o.N + i] =
              o.gru.set ? gv[i] : critic_value(o, run, ob.data() + size_t(i) * o.D);
      uint8_t d;
      step_env(o, run, env, s, act.data(), r.data(), &d);
      if (d && o.gru.set) std::fill_n(&o.hidden[ge * o.N * GRU_H], size_t(o.N) * GRU_H, 0.0);   // new episode
      if (rew_traj) std::memcpy(rew_traj + (size_t(t) * TE + ge) * RW, r.data(), RW * sizeof(double));
      if (done_traj) done_traj[size_t(t) * TE + ge] = d;
    }
    if (last_obs) observe_env(o, ge, last_obs + ge * row);
    if (last_value) {
      observe_env(o, ge, ob.data());
      for (int i = 0; i < o.N; ++i) {
        if (o.gru.set) {
          // one more evaluation on a copy of the carried state
          std::vector<double> hcopy(&o.hidden[(ge * o.N + i) * GRU_H], &o.hidden[(ge * o.N + i) * GRU_H] + GRU_H);
          double z[NUM_ACTIONS];
          gru_forward(o, run, ob.data() + size_t(i) * o.D, hcopy.data(), z, &last_value[ge * o.N + i]);
        } else {
          last_value[ge * o.N + i] = critic_value(o, run, ob.data() + size_t(i) * o.D);
        }
      }
    }
  }
}

thread_local std::string g_err;
int fail(const char* msg) { g_err = msg; return -1; }

}  // namespace

// =====================================================================================
// C interface (host pointers only).  Returns 0 on success, -1 on error.
// =====================================================================================
extern "C" {

struct orc_config {
  int32_t num_envs, num_agents, num_landmarks, num_runs, max_episode_steps;
  int32_t hidden, weight_dtype;
  int32_t env_offset, run_offset;
  double dt, damping, mass, accel;
  double agent_radius, landmark_radius;
  double contact_force, contact_margin;
  int32_t reward_mode;
  int32_t reserved;
  double local_ratio;
  int32_t scenario;
  int32_t num_adversaries;
  double adv_radius, adv_accel, adv_max_speed, good_max_speed;
};

const char* orc_last_error(void) { return g_err.c_str(); }

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

int orc_create(const orc_config* c, void** out) {
  if (!c || !out) return fail("null argument");
  if (c->scenario != 0 && c->scenario != 1) return fail("scenario must be 0 or 1");
  if (c->num_envs < 1 || c->num_agents < 1 || c->num_landmarks < (c->scenario == 1 ? 0 : 1) || c->num_runs < 1 ||
      c->max_episode_steps < 1)
    return fail("sizes must be positive");
  if (c->reward_mode != 0 && c->reward_mode != 1) return fail("reward_mode must be 0 or 1");
  if (c->scenario == 1 && (c->num_adversaries < 1 || c->num_adversaries >= c->num_agents))
    return fail("scenario 1 needs 1 <= num_adversaries < num_agents");
  static_assert(sizeof(orc_config) == sizeof(Config), "config mirror");
  Oracle* o = new Oracle();
  std::memcpy(&o->cfg, c, sizeof(Config));
  o->E = c->num_envs; o->N = c->num_agents; o->L = c->num_landmarks; o->R = c->num_runs;
  o->D = c->scenario == 1 ? 4 + 2 * o->L + 2 * (o->N - 1) + 2 * (o->N - c->num_adversaries)
                          : 4 + 2 * o->L + 4 * (o->N - 1);
  o->H = c->hidden;
  const size_t TE = size_t(o->R) * o->E;
  o->pos_a.assign(TE * o->N * 2, 0.0);
  o->vel_a.assign(TE * o->N * 2, 0.0);
  o->pos_l.assign(TE * o->L * 2, 0.0);
  o->ep_step.assign(TE, 0);
  o->hidden.assign(TE * o->N * GRU_H, 0.0);
  *out = o;
  return 0;
}

int orc_destroy(void* h) { delete static_cast<Oracle*>(h); return 0; }

int orc_set_threads(void* h, int n) {
  if (!h || n < 1) return fail("bad thread count");
  static_cast<Oracle*>(h)->nthreads = n;
  return 0;
}

int orc_obs_dim(void* h) { return static_cast<Oracle*>(h)->D; }

// obs: [R*E][N][D] doubles, may be null.
int orc_observe(void* h, double* obs) {
  Oracle& o = *static_cast<Oracle*>(h);
  const size_t TE = size_t(o.R) * o.E;
  for (size_t ge = 0; ge < TE; ++ge) observe_env(o, ge, obs + ge * o.N * o.D);
  return 0;
}

int orc_reset(void* h, uint32_t seed, double* obs) {
  if (!h) return fail("null handle");
  Oracle& o = *static_cast<Oracle*>(h);
  o.seed = seed;
  o.abs_step = 0;
  for (int run = 0; run < o.R; ++run)
    for (int env = 0; env < o.E; ++env) reset_env(o, run, env, 0);
  std::fill(o.hidden.begin(), o.hidden.end(), 0.0);
  o.was_reset = true;
  if (obs) orc_observe(h, obs);
  return 0;
}

// actions: [R*E][N]; obs [R*E][N][D] (nullable); reward [R*E] ([R*E][N] in reward_mode 1); done [R*E].
int orc_step(void* h, const uint8_t* actions, double* obs, double* reward, uint8_t* done) {
  if (!h || !actions) return fail("null argument");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.was_reset) return fail("step before reset");
  const size_t TE = size_t(o.R) * o.E;
  for (size_t ge = 0; ge < TE; ++ge) {
    for (int i = 0; i < o.N; ++i)
      if (actions[ge * o.N + i] >= NUM_ACTIONS) return fail("action out of range");
  }
  const size_t RW = (o.cfg.reward_mode == 1 || o.cfg.scenario == 1) ? size_t(o.N) : 1;
  std::vector<double> r(RW);
  for (size_t ge = 0; ge < TE; ++ge) {
    uint8_t d;
    step_env(o, int(ge / o.E), int(ge % o.E), o.abs_step, actions + ge * o.N, r.data(), &d);
    if (reward) std::memcpy(reward + ge * RW, r.data(), RW * sizeof(double));
    if (done) done[ge] = d;
  }
  o.abs_step += 1;
  if (obs) orc_observe(h, obs);
  return 0;
}

// Weights as float32, [R] leading dimension; layouts W1[D][H] b1[H] W2[H][H] b2[H] W3[H][5] b3[5].
// All six null => no policy (uniform random actions).
int orc_set_policy(void* h, const float* W1, const float* b1, const float* W2, const float* b2,
                   const float* W3, const float* b3) {
  if (!h) return fail("null handle");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!W1 && !b1 && !W2 && !b2 && !W3 && !b3) { o.pol.set = false; return 0; }
  if (!W1 || !b1 || !W2 || !b2 || !W3 || !b3) return fail("all six policy arrays or none");
  if (o.H < 1) return fail("hidden width not set");
  const bool bf = o.cfg.weight_dtype == 1;
  auto load = [&](std::vector<double>& dst, const float* src, size_t n, bool round_it) {
    dst.resize(n);
    for (size_t i = 0; i < n; ++i) dst[i] = round_it ? round_to_bf16(double(src[i])) : double(src[i]);
  };
  const size_t R = o.R, D = o.D, H = o.H;
  load(o.pol.W1, W1, R * D * H, bf);
  load(o.pol.b1, b1, R * H, false);
  load(o.pol.W2, W2, R * H * H, bf);
  load(o.pol.b2, b2, R * H, false);
  load(o.pol.W3, W3, R * H * NUM_ACTIONS, bf);
  load(o.pol.b3, b3, R * NUM_ACTIONS, false);
  o.pol.set = true;
  return 0;
}

// Critic weights as float32, [R] leading dimension: V1[D][H] c1[H] V2[H][H] c2[H] V3[H] c3[1].
// All six null => no critic.
int orc_set_critic(void* h, const float* V1, const float* c1, const float* V2, const float* c2,
                   const float* V3, const float* c3) {
  if (!h) return fail("null handle");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!V1 && !c1 && !V2 && !c2 && !V3 && !c3) { o.critic.set = false; return 0; }
  if (!V1 || !c1 || !V2 || !c2 || !V3 || !c3) return fail("all six critic arrays or none");
  if (o.H < 1) return fail("hidden width not set");
  const bool bf = o.cfg.weight_dtype == 1;
  auto load = [&](std::vector<double>& dst, const float* src, size_t n, bool round_it) {
    dst.resize(n);
    for (size_t i = 0; i < n; ++i) dst[i] = round_it ? round_to_bf16(double(src[i])) : double(src[i]);
  };
  const size_t R = o.R, D = o.D, H = o.H;
  load(o.critic.W1, V1, R * D * H, bf);
  load(o.critic.b1, c1, R * H, false);
  load(o.critic.W2, V2, R * H * H, bf);
  load(o.critic.b2, c2, R * H, false);
  load(o.critic.W3, V3, R * H, bf);
  load(o.critic.b3, c3, R, false);
  o.critic.set = true;
  return 0;
}

// Recurrent policy (R-15) weights as float32, [R] leading dimension: We[D][128] be[128] Wi[128][384]
// bi[384] Wh[128][384] bh[384] Wf[128][128] bf[128] Wo[128][5] bo[5].  All ten null => removed.
int orc_set_gru(void* h, const float* We, const float* be, const float* Wi, const float* bi, const float* Wh,
                const float* bh, const float* Wf, const float* bf, const float* Wo, const float* bo) {
  if (!h) return fail("null handle");
  Oracle& o = *static_cast<Oracle*>(h);
  const float* all[10] = {We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo};
  int given = 0;
  for (const float* p : all) given += p != nullptr;
  if (given == 0) { o.gru.set = false; return 0; }
  if (given != 10) return fail("all ten recurrent-policy arrays or none");
  const bool b16 = o.cfg.weight_dtype == 1;
  auto load = [&](std::vector<double>& dst, const float* src, size_t n, bool round_it) {
    dst.resize(n);
    for (size_t i = 0; i < n; ++i) dst[i] = round_it ? round_to_bf16(double(src[i])) : double(src[i]);
  };
  const size_t R = o.R, D = o.D, G = GRU_H;
  load(o.gru.We, We, R * D * G, b16);
  load(o.gru.be, be, R * G, false);
  load(o.gru.Wi, Wi, R * G * 3 * G, b16);
  load(o.gru.bi, bi, R * 3 * G, false);
  load(o.gru.Wh, Wh, R * G * 3 * G, b16);
  load(o.gru.bh, bh, R * 3 * G, false);
  load(o.gru.Wf, Wf, R * G * G, b16);
  load(o.gru.bf, bf, R * G, false);
  load(o.gru.Wo, Wo, R * G * NUM_ACTIONS, b16);
  load(o.gru.bo, bo, R * NUM_ACTIONS, false);
  o.gru.set = true;
  return 0;
}

// Critic head of the recurrent actor-critic (R-16) as float32, [R] leading dimension: Wc[128][128] bc[128]
// wv[128] bv[1].  All four null => removed.
int orc_set_gru_critic(void* h, const float* Wc, const float* bc, const float* wv, const float* bv) {
  if (!h) return fail("null handle");
  Oracle& o = *static_cast<Oracle*>(h);
  const int given = (Wc != nullptr) + (bc != nullptr) + (wv != nullptr) + (bv != nullptr);
  if (given == 0) { o.gru_critic.set = false; return 0; }
  if (given != 4) return fail("all four critic-head arrays or none");
  const bool b16 = o.cfg.weight_dtype == 1;
  auto load = [&](std::vector<double>& dst, const float* src, size_t n, bool round_it) {
    dst.resize(n);
    for (size_t i = 0; i < n; ++i) dst[i] = round_it ? round_to_bf16(double(src[i])) : double(src[i]);
  };
  const size_t R = o.R, G = GRU_H;
  load(o.gru_critic.Wc, Wc, R * G * G, b16);
  load(o.gru_critic.bc, bc, R * G, false);
  load(o.gru_critic.wv, wv, R * G, b16);
  load(o.gru_critic.bv, bv, R, false);
  o.gru_critic.set = true;
  return 0;
}

// One recurrent-policy evaluation per row: obs [n][D], hidden [n][128] in/out, logits [n][5]; values [n]
// (nullable) the critic head of R-16 on the new hidden state.
int orc_gru_forward(void* h, int run, const double* obs, int n, double* hidden, double* logits, double* values) {
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.gru.set) return fail("no recurrent policy");
  if (values && !o.gru_critic.set) return fail("no recurrent critic head");
  if (run < 0 || run >= o.R) return fail("bad run");
  for (int r = 0; r < n; ++r)
    gru_forward(o, run, obs + size_t(r) * o.D, hidden + size_t(r) * GRU_H, logits + size_t(r) * NUM_ACTIONS,
                values ? values + r : nullptr);
  return 0;
}

// Hidden state [R*E][N][128]; orc_set_hidden(null) zeroes it.
int orc_get_hidden(void* h, double* hidden) {
  Oracle& o = *static_cast<Oracle*>(h);
  std::memcpy(hidden, o.hidden.data(), o.hidden.size() * sizeof(double));
  return 0;
}
int orc_set_hidden(void* h, const double* hidden) {
  Oracle& o = *static_cast<Oracle*>(h);
  if (hidden) std::memcpy(o.hidden.data(), hidden, o.hidden.size() * sizeof(double));
  else std::fill(o.hidden.begin(), o.hidden.end(), 0.0);
  return 0;
}

// Critic values of `run` for n observation rows [n][D] -> [n].
int orc_value(void* h, int run, const double* obs, int n, double* values) {
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.critic.set) return fail("no critic");
  if (run < 0 || run >= o.R) return fail("bad run");
  for (int r = 0; r < n; ++r) values[r] = critic_value(o, run, obs + size_t(r) * o.D);
  return 0;
}

// log pi(k | logits) for all five actions.
void orc_log_probs(const double* logits, double* lp) { log_probs(logits, lp); }

// Logits of the policy of `run` for n observation rows [n][D] -> [n][5].
int orc_policy_logits(void* h, int run, const double* obs, int n, double* logits) {
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.pol.set) return fail("no policy");
  if (run < 0 || run >= o.R) return fail("bad run");
  for (int r = 0; r < n; ++r) policy_logits(o, run, obs + size_t(r) * o.D, logits + size_t(r) * NUM_ACTIONS);
  return 0;
}

int orc_gumbel_max_action(uint32_t seed, uint32_t run, uint32_t env, uint32_t step, uint32_t agent,
                          const double* logits) {
  return gumbel_max_action(seed, run, env, step, agent, logits);
}

int orc_uniform_action(uint32_t seed, uint32_t run, uint32_t env, uint32_t step, uint32_t agent) {
  return uniform_action(seed, run, env, step, agent);
}

double orc_round_to_bf16(double x) { return round_to_bf16(x); }

int orc_rollout(void* h, int32_t T, double* obs_traj, uint8_t* act_traj, double* rew_traj,
                uint8_t* done_traj, double* last_obs) {
  if (!h || T < 1) return fail("bad argument");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.was_reset) return fail("rollout before reset");
  const size_t TE = size_t(o.R) * o.E;
  const int nt = int(std::min<size_t>(size_t(o.nthreads), TE));
  if (nt <= 1) {
    rollout_range(o, 0, TE, T, obs_traj, act_traj, rew_traj, done_traj, last_obs);
  } else {
    // Envs are independent: contiguous env ranges on separate threads, same arithmetic.
    std::vector<std::thread> th;
    for (int k = 0; k < nt; ++k) {
      const size_t g0 = TE * k / nt, g1 = TE * (k + 1) / nt;
      th.emplace_back([&, g0, g1] {
        rollout_range(o, g0, g1, T, obs_traj, act_traj, rew_traj, done_traj, last_obs);
      });
    }
    for (auto& t : th) t.join();
  }
  o.abs_step += uint32_t(T);
  return 0;
}

// Actor-critic rollout: orc_rollout plus logp_traj, value_traj [T][R*E][N] and last_value [R*E][N].
int orc_rollout_ac(void* h, int32_t T, double* obs_traj, uint8_t* act_traj, double* logp_traj,
                   double* value_traj, double* rew_traj, uint8_t* done_traj, double* last_obs,
                   double* last_value) {
  if (!h || T < 1) return fail("bad argument");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!o.was_reset) return fail("rollout before reset");
  if (o.gru.set) {
    if (!o.gru_critic.set) return fail("actor-critic rollout with the recurrent policy needs its critic head");
  } else if (!o.pol.set || !o.critic.set) {
    return fail("actor-critic rollout needs a policy and a critic");
  }
  const size_t TE = size_t(o.R) * o.E;
  const int nt = int(std::max<size_t>(1, std::min<size_t>(size_t(o.nthreads), TE)));
  std::vector<std::thread> th;
  for (int k = 0; k < nt; ++k) {
    const size_t g0 = TE * k / nt, g1 = TE * (k + 1) / nt;
    th.emplace_back([&, g0, g1] {
      rollout_range(o, g0, g1, T, obs_traj, act_traj, rew_traj, done_traj, last_obs, logp_traj, value_traj,
                    last_value);
    });
  }
  for (auto& t : th) t.join();
  o.abs_step += uint32_t(T);
  return 0;
}

// State in the oracle's own layout: pos_a, vel_a [R*E][N][2]; pos_l [R*E][L][2]; ep_step [R*E].
int orc_get_state(void* h, double* pos_a, double* vel_a, double* pos_l, int32_t* ep_step,
                  uint32_t* abs_step) {
  Oracle& o = *static_cast<Oracle*>(h);
  // (a scenario without landmarks has an empty pos_l: nothing to copy, and no pointer to copy from)
  if (pos_a) std::memcpy(pos_a, o.pos_a.data(), o.pos_a.size() * sizeof(double));
  if (vel_a) std::memcpy(vel_a, o.vel_a.data(), o.vel_a.size() * sizeof(double));
  if (pos_l && !o.pos_l.empty()) std::memcpy(pos_l, o.pos_l.data(), o.pos_l.size() * sizeof(double));
  if (ep_step) std::memcpy(ep_step, o.ep_step.data(), o.ep_step.size() * sizeof(int32_t));
  if (abs_step) *abs_step = o.abs_step;
  return 0;
}

int orc_set_state(void* h, const double* pos_a, const double* vel_a, const double* pos_l,
                  const int32_t* ep_step, uint32_t seed, uint32_t abs_step) {
  if (!h || !pos_a || !vel_a || !ep_step) return fail("null argument");
  Oracle& o = *static_cast<Oracle*>(h);
  if (!pos_l && !o.pos_l.empty()) return fail("null argument");
  std::memcpy(o.pos_a.data(), pos_a, o.pos_a.size() * sizeof(double));
  std::memcpy(o.vel_a.data(), vel_a, o.vel_a.size() * sizeof(double));
  if (!o.pos_l.empty()) std::memcpy(o.pos_l.data(), pos_l, o.pos_l.size() * sizeof(double));
  std::memcpy(o.ep_step.data(), ep_step, o.ep_step.size() * sizeof(int32_t));
  o.seed = seed;
  o.abs_step = abs_step;
  o.was_reset = true;
  return 0;
}

}  // extern "C"
