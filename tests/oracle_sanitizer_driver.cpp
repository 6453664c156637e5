// Stand-alone driver for the oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only,
// compiled and run by tests/test_oracle_sanitizers.py).  It walks every entry point of the oracle over the
// shapes the parity tests use -- 1, 3 and 10 agents, several runs, threads, both scenarios (the second one
// also without landmarks), both reward modes, fp32 and bf16 policies, critic, recurrent policy, state in and
// out, rollouts that cross auto-resets -- and returns 0.  The sanitizers abort on any finding.
#include "../oracle/mpe_oracle.cpp"

#include <cstdio>
#include <cstdlib>

namespace {

struct Lcg {   // plain input generator for weights and actions (not the method's arithmetic)
  uint64_t s;
  float next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return float(int32_t(s >> 33) % 2001) / 2000.0f - 0.5f; }
};

#define OK(call) do { if ((call) != 0) { std::fprintf(stderr, "%s failed: %s\n", #call, orc_last_error()); std::exit(3); } } while (0)

std::vector<float> fill(Lcg& g, size_t n) {
  std::vector<float> v(n);
  for (float& x : v) x = g.next();
  return v;
}

void exercise(int scenario, int E, int N, int L, int R, int H, int wd, int reward_mode, int threads, bool gru, bool critic) {
  orc_config c{};
  c.num_envs = E; c.num_agents = N; c.num_landmarks = L; c.num_runs = R; c.max_episode_steps = 7;
  c.hidden = H; c.weight_dtype = wd; c.env_offset = 3; c.run_offset = 2;
  c.dt = 0.1; c.damping = 0.25; c.mass = 1.0; c.accel = scenario ? 4.0 : 5.0;
  c.agent_radius = scenario ? 0.05 : 0.15; c.landmark_radius = scenario ? 0.2 : 0.05;
  c.contact_force = 100.0; c.contact_margin = 1e-3; c.reward_mode = reward_mode; c.local_ratio = 0.5;
  c.scenario = scenario; c.num_adversaries = scenario ? N - 1 : 0;
  c.adv_radius = 0.075; c.adv_accel = 3.0; c.adv_max_speed = 1.0; c.good_max_speed = 1.3;
  void* h = nullptr;
  OK(orc_create(&c, &h));
  OK(orc_set_threads(h, threads));
  const size_t TE = size_t(R) * E, D = size_t(orc_obs_dim(h));
  const size_t RW = (reward_mode == 1 || scenario == 1) ? size_t(N) : 1;
  Lcg g{uint64_t(E * 131 + N * 17 + scenario)};
  if (H && !gru) {
    auto W1 = fill(g, R * D * H), b1 = fill(g, size_t(R) * H), W2 = fill(g, size_t(R) * H * H), b2 = fill(g, size_t(R) * H),
         W3 = fill(g, size_t(R) * H * 5), b3 = fill(g, size_t(R) * 5);
    OK(orc_set_policy(h, W1.data(), b1.data(), W2.data(), b2.data(), W3.data(), b3.data()));
    if (critic) {
      auto V3 = fill(g, size_t(R) * H), c3 = fill(g, size_t(R));
      OK(orc_set_critic(h, W1.data(), b1.data(), W2.data(), b2.data(), V3.data(), c3.data()));
    }
  }
  if (gru) {
    const size_t G = 128;
    auto We = fill(g, R * D * G), be = fill(g, R * G), Wi = fill(g, R * G * 3 * G), bi = fill(g, R * 3 * G),
         Wh = fill(g, R * G * 3 * G), bh = fill(g, R * 3 * G), Wf = fill(g, R * G * G), bf = fill(g, R * G),
         Wo = fill(g, R * G * 5), bo = fill(g, size_t(R) * 5);
    OK(orc_set_gru(h, We.data(), be.data(), Wi.data(), bi.data(), Wh.data(), bh.data(), Wf.data(), bf.data(), Wo.data(), bo.data()));
  }
  std::vector<double> obs(TE * N * D), rew(TE * RW);
  std::vector<uint8_t> done(TE), act(TE * N);
  OK(orc_reset(h, 99u, obs.data()));
  for (int t = 0; t < 9; ++t) {   // single steps across an auto-reset
    for (uint8_t& a : act) a = uint8_t((g.next() + 0.5f) * 4.99f);
    OK(orc_step(h, act.data(), obs.data(), rew.data(), done.data()));
  }
  const int T = 17;
  std::vector<double> ot(size_t(T) * TE * N * D), rt(size_t(T) * TE * RW), last(TE * N * D);
  std::vector<uint8_t> at(size_t(T) * TE * N), dt(size_t(T) * TE);
  OK(orc_rollout(h, T, ot.data(), at.data(), rt.data(), dt.data(), last.data()));
  OK(orc_rollout(h, 3, nullptr, at.data(), rt.data(), dt.data(), nullptr));
  if (critic) {
    std::vector<double> lp(size_t(T) * TE * N), val(size_t(T) * TE * N), lv(TE * N);
    OK(orc_rollout_ac(h, T, ot.data(), at.data(), lp.data(), val.data(), rt.data(), dt.data(), last.data(), lv.data()));
    OK(orc_value(h, R - 1, obs.data(), int(N), lv.data()));
    std::vector<double> z(size_t(N) * 5);
    OK(orc_policy_logits(h, R - 1, obs.data(), int(N), z.data()));
    double l5[5];
    orc_log_probs(z.data(), l5);
  }
  if (gru) {
    std::vector<double> hid(TE * N * 128), z(size_t(N) * 5);
    OK(orc_get_hidden(h, hid.data()));
    OK(orc_set_hidden(h, hid.data()));
    OK(orc_gru_forward(h, 0, obs.data(), int(N), hid.data(), z.data(), nullptr));
    // the recurrent actor-critic: critic head, rollout with values, removal
    const size_t G = 128;
    auto Wc = fill(g, R * G * G), bc = fill(g, R * G), wv = fill(g, R * G), bv = fill(g, size_t(R));
    OK(orc_set_gru_critic(h, Wc.data(), bc.data(), wv.data(), bv.data()));
    std::vector<double> vals(N);
    OK(orc_gru_forward(h, R - 1, obs.data(), int(N), hid.data(), z.data(), vals.data()));
    std::vector<double> lp(size_t(T) * TE * N), val(size_t(T) * TE * N), lv(TE * N);
    OK(orc_rollout_ac(h, T, ot.data(), at.data(), lp.data(), val.data(), rt.data(), dt.data(), last.data(), lv.data()));
    OK(orc_rollout_ac(h, 2, nullptr, nullptr, nullptr, val.data(), nullptr, nullptr, nullptr, lv.data()));
    OK(orc_set_gru_critic(h, nullptr, nullptr, nullptr, nullptr));
    OK(orc_set_hidden(h, nullptr));
  }
  std::vector<double> pa(TE * N * 2), va(TE * N * 2), pl(TE * L * 2);
  std::vector<int32_t> ep(TE);
  uint32_t s = 0;
  OK(orc_get_state(h, pa.data(), va.data(), pl.data(), ep.data(), &s));
  OK(orc_set_state(h, pa.data(), va.data(), L ? pl.data() : nullptr, ep.data(), 5u, s));
  OK(orc_rollout(h, 8, ot.data(), at.data(), rt.data(), dt.data(), last.data()));
  OK(orc_observe(h, obs.data()));
  OK(orc_destroy(h));
}

}  // namespace

int main() {
  uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
  orc_philox4x32_10(ctr, key, out);
  double z[5] = {0.1, -0.2, 0.3, 0.0, 1.0};
  (void)orc_gumbel_max_action(1, 2, 3, 4, 5, z);
  (void)orc_uniform_action(1, 2, 3, 4, 5);
  exercise(0, 5, 1, 1, 1, 0, 0, 0, 1, false, false);
  exercise(0, 7, 3, 3, 2, 64, 0, 0, 3, false, true);
  exercise(0, 4, 3, 3, 1, 64, 1, 1, 2, false, true);
  exercise(0, 3, 10, 10, 1, 128, 1, 0, 2, false, false);
  exercise(0, 6, 10, 10, 2, 0, 0, 1, 4, false, false);
  exercise(0, 5, 3, 3, 2, 128, 1, 0, 2, true, false);
  exercise(1, 4, 4, 2, 1, 128, 0, 0, 3, true, false);   // recurrent policy on the second scenario
  exercise(1, 6, 4, 2, 1, 64, 0, 0, 2, false, true);
  exercise(1, 5, 3, 0, 2, 64, 1, 0, 1, false, false);   // no landmarks: empty pos_l
  exercise(1, 4, 6, 2, 1, 0, 0, 0, 3, false, false);
  exercise(1, 3, 2, 1, 1, 0, 0, 0, 8, false, false);    // more threads than envs
  std::puts("oracle sanitizer driver: ok");
  return 0;
}
