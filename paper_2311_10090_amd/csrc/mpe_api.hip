// C ABI of libmpe (see include/mpe.h): handle, host-side validation, dispatch to kernels.
#include "../../include/mpe.h"

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <new>

#include "mpe_launch.h"

using namespace mpe;

struct mpe_env {
  mpe_config cfg;
  int N = 0, D = 0, H = 0;
  int L = 0, G = 0;     // landmarks; good agents (tag scenario)
  bool tag = false;
  TagPhys tg{};
  uint32_t TE = 0, E = 0, R = 0;
  Phys ph{};
  StatePtrs st{};
  bool ready = false;  // reset or set_state has been called
  uint32_t seed = 0;
  uint32_t abs_step = 0;
  PolicyBuffers pol{};
  bool has_policy = false;
  PolicyBuffers critic{};
  bool has_critic = false;
  PolicyBuffers gru{};        // recurrent policy; takes precedence over `pol` while set
  bool has_gru = false;
  float* hidden = nullptr;    // [TE][N][128] carried state of the recurrent policy (allocated with it)
  PolicyBuffers gru_critic{}; // critic head of the recurrent actor-critic
  bool has_gru_critic = false;
  // One word of pinned host memory, mapped into the device: a kernel whose bounded wait gave up raises it
  // (see group_barrier); the host reads it, without any synchronisation, at the start of the next call.
  uint32_t* fault_host = nullptr;
  uint32_t* fault_dev = nullptr;
  uint32_t barrier_polls = 1u << 24;   // see mpe_set_barrier_poll_limit
};

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define MPE_HIP(call)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) return fail(MPE_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool finite_pos(float v) { return std::isfinite(v) && v > 0.0f; }

int validate(const mpe_config* c) {
  if (c->num_envs < 1) return fail(MPE_EINVAL, "num_envs must be >= 1 (got %d)", c->num_envs);
  if (c->num_runs < 1) return fail(MPE_EINVAL, "num_runs must be >= 1 (got %d)", c->num_runs);
  if (c->num_agents < 1 || c->num_agents > MPE_MAX_AGENTS)
    return fail(MPE_EINVAL, "num_agents must be in [1, %d] (got %d)", MPE_MAX_AGENTS, c->num_agents);
  if (c->scenario != MPE_SCENARIO_SPREAD && c->scenario != MPE_SCENARIO_TAG)
    return fail(MPE_EINVAL, "scenario must be MPE_SCENARIO_SPREAD or MPE_SCENARIO_TAG (got %d)", c->scenario);
  if (c->scenario == MPE_SCENARIO_SPREAD && c->num_landmarks != c->num_agents)
    return fail(MPE_EINVAL, "simple-spread needs num_landmarks == num_agents (got %d, %d)",
                c->num_landmarks, c->num_agents);
  if (c->scenario == MPE_SCENARIO_TAG) {
    if (c->num_adversaries < 1 || c->num_adversaries >= c->num_agents)
      return fail(MPE_EINVAL, "MPE_SCENARIO_TAG needs 1 <= num_adversaries < num_agents (got %d, %d)",
                  c->num_adversaries, c->num_agents);
    if (!tag_supported(c->num_agents, c->num_landmarks, c->num_agents - c->num_adversaries))
      return fail(MPE_EINVAL, "MPE_SCENARIO_TAG is built for (agents, landmarks, good agents) in "
                              "{(4,2,1), (2,1,1), (3,0,1), (6,2,2)} (got %d, %d, %d)",
                  c->num_agents, c->num_landmarks, c->num_agents - c->num_adversaries);
    if (!std::isfinite(c->adv_radius) || c->adv_radius < 0.0f || !std::isfinite(c->adv_accel))
      return fail(MPE_EINVAL, "adv_radius must be finite and >= 0, adv_accel finite");
    if (!finite_pos(c->adv_max_speed) || !finite_pos(c->good_max_speed))
      return fail(MPE_EINVAL, "adv_max_speed and good_max_speed must be finite and > 0");
  }
  const uint64_t te = uint64_t(c->num_envs) * uint64_t(c->num_runs);
  if (te > (1ull << 30)) return fail(MPE_EINVAL, "num_envs * num_runs must be <= 2^30");
  if (c->max_episode_steps < 1) return fail(MPE_EINVAL, "max_episode_steps must be >= 1");
  if (!finite_pos(c->dt) || !finite_pos(c->mass) || !finite_pos(c->contact_margin))
    return fail(MPE_EINVAL, "dt, mass and contact_margin must be finite and > 0");
  if (!std::isfinite(c->damping) || c->damping < 0.0f || c->damping > 1.0f)
    return fail(MPE_EINVAL, "damping must be in [0, 1]");
  if (!std::isfinite(c->accel) || !std::isfinite(c->contact_force) || !std::isfinite(c->agent_radius) ||
      !std::isfinite(c->landmark_radius) || c->agent_radius < 0.0f || c->landmark_radius < 0.0f)
    return fail(MPE_EINVAL, "accel, contact_force and radii must be finite, radii >= 0");
  if (c->hidden != 0 && c->hidden != 64 && c->hidden != 128)
    return fail(MPE_EINVAL, "hidden must be 0 (no policy), 64 or 128 (got %d)", c->hidden);
  if (c->weight_dtype != MPE_WEIGHTS_FP32 && c->weight_dtype != MPE_WEIGHTS_BF16)
    return fail(MPE_EINVAL, "weight_dtype must be MPE_WEIGHTS_FP32 or MPE_WEIGHTS_BF16");
  if (c->reward_mode != MPE_REWARD_SHARED && c->reward_mode != MPE_REWARD_MIXED)
    return fail(MPE_EINVAL, "reward_mode must be MPE_REWARD_SHARED or MPE_REWARD_MIXED");
  if (c->reward_mode == MPE_REWARD_MIXED &&
      (!std::isfinite(c->local_ratio) || c->local_ratio < 0.0f || c->local_ratio > 1.0f))
    return fail(MPE_EINVAL, "local_ratio must be in [0, 1]");
  return MPE_OK;
}

size_t agent_floats(const mpe_env* e) { return size_t(2) * e->N * e->TE; }
size_t landmark_floats(const mpe_env* e) { return size_t(2) * e->L * e->TE; }

// Fill the host-side fields of a handle from a validated config (no device work).
void init_from_config(mpe_env* e, const mpe_config* cfg) {
  e->cfg = *cfg;
  e->N = cfg->num_agents;
  e->L = cfg->num_landmarks;
  e->tag = cfg->scenario == MPE_SCENARIO_TAG;
  e->G = e->tag ? e->N - cfg->num_adversaries : 0;
  e->D = e->tag ? 4 + 2 * e->L + 2 * (e->N - 1) + 2 * e->G : 6 * e->N;
  e->H = cfg->hidden;
  e->E = uint32_t(cfg->num_envs);
  e->R = uint32_t(cfg->num_runs);
  e->TE = e->E * e->R;
  // Combine constants in double, round once.
  e->ph.dt = cfg->dt;
  e->ph.keep = float(1.0 - double(cfg->damping));
  e->ph.dt_over_mass = float(double(cfg->dt) / double(cfg->mass));
  e->ph.accel = cfg->accel;
  e->ph.two_r = float(2.0 * double(cfg->agent_radius));
  e->ph.inv_margin = float(1.0 / double(cfg->contact_margin));
  e->ph.force_margin = float(double(cfg->contact_force) * double(cfg->contact_margin));
  e->ph.max_ep = cfg->max_episode_steps;
  e->ph.reward_mode = cfg->reward_mode;
  e->ph.local_ratio = cfg->reward_mode == MPE_REWARD_MIXED ? cfg->local_ratio : 0.0f;
  e->ph.two_r_sq = float(4.0 * double(cfg->agent_radius) * double(cfg->agent_radius));
  if (e->tag) {
    TagPhys& t = e->tg;
    t.dt = cfg->dt;
    t.keep = e->ph.keep;
    t.dt_over_mass = e->ph.dt_over_mass;
    t.inv_margin = e->ph.inv_margin;
    t.force_margin = e->ph.force_margin;
    t.max_ep = cfg->max_episode_steps;
    t.radius[0] = cfg->adv_radius;
    t.radius[1] = cfg->agent_radius;
    t.gain[0] = cfg->adv_accel;
    t.gain[1] = cfg->accel;
    t.limit[0] = cfg->adv_max_speed;
    t.limit[1] = cfg->good_max_speed;
    t.limit_sq[0] = float(double(cfg->adv_max_speed) * double(cfg->adv_max_speed));
    t.limit_sq[1] = float(double(cfg->good_max_speed) * double(cfg->good_max_speed));
    t.lm_radius = cfg->landmark_radius;
    const double touch = double(cfg->adv_radius) + double(cfg->agent_radius);
    t.touch_sq = float(touch * touch);
  }
}

// A kernel of an earlier call on this handle gave up a bounded wait: its results, and the state it wrote
// back, are invalid.
int check_fault(const mpe_env* e, const char* who) {
  if (e->fault_host && *static_cast<volatile const uint32_t*>(e->fault_host) != 0u)
    return fail(MPE_EHIP, "%s: a kernel of an earlier call on this handle gave up waiting at a wavefront barrier; "
                          "the handle's state is invalid (destroy it)", who);
  return MPE_OK;
}

RolloutArgs rollout_args(const mpe_env* e, int32_t T, float* obs_traj, uint8_t* act_traj, float* rew_traj,
                         uint8_t* done_traj, float* last_obs) {
  RolloutArgs A;
  A.st = e->st;
  A.ph = e->ph;
  A.TE = e->TE;
  A.E = e->E;
  A.seed = e->seed;
  A.abs_step = e->abs_step;
  A.T = T;
  A.obs_traj = obs_traj;
  A.act_traj = act_traj;
  A.rew_traj = rew_traj;
  A.done_traj = done_traj;
  A.last_obs = last_obs;
  A.fault = e->fault_dev;
  A.barrier_polls = e->barrier_polls;
  return A;
}

}  // namespace

extern "C" {

const char* mpe_last_error(void) { return g_err; }

int mpe_create(const mpe_config* cfg, mpe_env** out) {
  if (!cfg || !out) return fail(MPE_EINVAL, "mpe_create: NULL argument");
  *out = nullptr;
  if (int rc = validate(cfg)) return rc;
  mpe_env* e = new (std::nothrow) mpe_env();
  if (!e) return fail(MPE_EHIP, "out of host memory");
  init_from_config(e, cfg);
  const size_t nf = agent_floats(e) * sizeof(float);
  hipError_t err = hipMalloc(&e->st.pos_a, nf);
  if (err == hipSuccess) err = hipMalloc(&e->st.vel_a, nf);
  if (err == hipSuccess) err = hipMalloc(&e->st.pos_l, landmark_floats(e) * sizeof(float) + 16);
  if (err == hipSuccess) err = hipMalloc(&e->st.ep_step, size_t(e->TE) * sizeof(int32_t));
  if (err == hipSuccess) err = hipHostMalloc(reinterpret_cast<void**>(&e->fault_host), sizeof(uint32_t), hipHostMallocMapped);
  if (err == hipSuccess) {
    *e->fault_host = 0u;
    err = hipHostGetDevicePointer(reinterpret_cast<void**>(&e->fault_dev), e->fault_host, 0);
  }
  if (err != hipSuccess) {
    int rc = fail(MPE_EHIP, "mpe_create: allocation failed: %s", hipGetErrorString(err));
    (void)hipFree(e->st.pos_a); (void)hipFree(e->st.vel_a); (void)hipFree(e->st.pos_l); (void)hipFree(e->st.ep_step);
    if (e->fault_host) (void)hipHostFree(e->fault_host);
    delete e;
    return rc;
  }
  *out = e;
  return MPE_OK;
}

int mpe_destroy(mpe_env* e) {
  if (!e) return MPE_OK;
  (void)hipDeviceSynchronize();
  (void)hipFree(e->st.pos_a);
  (void)hipFree(e->st.vel_a);
  (void)hipFree(e->st.pos_l);
  (void)hipFree(e->st.ep_step);
  free_policy(e->pol);
  free_policy(e->critic);
  free_policy(e->gru);
  free_policy(e->gru_critic);
  if (e->hidden) (void)hipFree(e->hidden);
  if (e->fault_host) (void)hipHostFree(e->fault_host);
  delete e;
  return MPE_OK;
}

int mpe_obs_dim(const mpe_env* e) {
  if (!e) return fail(MPE_EINVAL, "mpe_obs_dim: NULL handle");
  return e->D;
}

int mpe_reset(mpe_env* e, uint32_t seed, float* obs, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_reset: NULL handle");
  if (obs && !aligned16(obs)) return fail(MPE_EINVAL, "mpe_reset: obs must be 16-byte aligned");
  if (e->tag) launch_tag_reset(e->N, e->L, e->G, e->st, e->TE, e->E, seed, obs, static_cast<hipStream_t>(stream));
  else launch_reset(e->N, e->st, e->TE, e->E, seed, obs, static_cast<hipStream_t>(stream));
  if (e->hidden) launch_fill_zero(e->hidden, size_t(e->TE) * e->N * 128, static_cast<hipStream_t>(stream));
  MPE_HIP(hipGetLastError());
  e->seed = seed;
  e->abs_step = 0;
  e->ready = true;
  return MPE_OK;
}

int mpe_step(mpe_env* e, const uint8_t* actions, float* obs, float* reward, uint8_t* done, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_step: NULL handle");
  if (!actions) return fail(MPE_EINVAL, "mpe_step: actions is NULL");
  if (!e->ready) return fail(MPE_ESTATE, "mpe_step: call mpe_reset or mpe_set_state first");
  if (int rc = check_fault(e, "mpe_step")) return rc;
  if ((obs && !aligned16(obs)) || (reward && !aligned16(reward)))
    return fail(MPE_EINVAL, "mpe_step: obs and reward must be 16-byte aligned");
  if (e->abs_step == 0xFFFFFFFFu) return fail(MPE_EINVAL, "mpe_step: absolute step counter would overflow 32 bits");
  if (e->tag) {
    TagArgs A{};
    A.r.st = e->st;
    A.r.TE = e->TE;
    A.r.E = e->E;
    A.r.seed = e->seed;
    A.r.abs_step = e->abs_step;
    A.r.T = 1;
    A.r.rew_traj = reward;
    A.r.done_traj = done;
    A.r.last_obs = obs;
    A.r.fault = e->fault_dev;
    A.tg = e->tg;
    A.actions_in = actions;
    const char* why = nullptr;
    hipError_t err = launch_tag_rollout(e->N, e->L, e->G, 0, A, nullptr, nullptr, static_cast<hipStream_t>(stream), &why);
    if (why) return fail(MPE_EINVAL, "mpe_step: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_step: %s", hipGetErrorString(err));
  } else {
    launch_step(e->N, e->st, e->ph, e->TE, e->E, e->seed, e->abs_step, actions, obs, reward, done,
                static_cast<hipStream_t>(stream));
  }
  MPE_HIP(hipGetLastError());
  e->abs_step += 1;
  return MPE_OK;
}

int mpe_set_policy(mpe_env* e, const float* W1, const float* b1, const float* W2, const float* b2,
                   const float* W3, const float* b3, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_policy: NULL handle");
  const int given = (W1 != nullptr) + (b1 != nullptr) + (W2 != nullptr) + (b2 != nullptr) +
                    (W3 != nullptr) + (b3 != nullptr);
  if (given == 0) {
    e->has_policy = false;
    return MPE_OK;
  }
  if (given != 6) return fail(MPE_EINVAL, "mpe_set_policy: pass all six arrays or none");
  if (e->H != 64 && e->H != 128) return fail(MPE_EINVAL, "mpe_set_policy: config.hidden must be 64 or 128");
  const char* why = nullptr;
  hipError_t err;
  e->has_policy = false;   // a failure below must not leave an earlier policy installed on a partly rewritten buffer
  if (e->tag) {
    if (!tag_policy_supported(e->N, e->L, e->G, e->H, e->cfg.weight_dtype))
      return fail(MPE_EINVAL, "mpe_set_policy: MPE_SCENARIO_TAG policies are built for hidden 64 and observation "
                              "rows of at most 32 floats");
    err = pack_policy_tag(e->pol, e->N, e->L, e->G, int(e->R), e->cfg.weight_dtype == MPE_WEIGHTS_BF16, 5, W1, b1, W2,
                          b2, W3, b3, static_cast<hipStream_t>(stream));
  } else {
    err = pack_policy(e->pol, e->N, e->H, int(e->R), e->cfg.weight_dtype, W1, b1, W2, b2, W3, b3,
                      static_cast<hipStream_t>(stream), &why);
  }
  if (why) return fail(MPE_EINVAL, "mpe_set_policy: %s", why);
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_set_policy: %s", hipGetErrorString(err));
  e->has_policy = true;
  return MPE_OK;
}

int mpe_rollout(mpe_env* e, int32_t T, float* obs_traj, uint8_t* act_traj, float* rew_traj,
                uint8_t* done_traj, float* last_obs, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_rollout: NULL handle");
  if (T < 1 || T > MPE_MAX_ROLLOUT_STEPS)
    return fail(MPE_EINVAL, "mpe_rollout: T must be in [1, %d] (got %d)", MPE_MAX_ROLLOUT_STEPS, T);
  if (!e->ready) return fail(MPE_ESTATE, "mpe_rollout: call mpe_reset or mpe_set_state first");
  if (int rc = check_fault(e, "mpe_rollout")) return rc;
  if ((obs_traj && !aligned16(obs_traj)) || (rew_traj && !aligned16(rew_traj)) ||
      (last_obs && !aligned16(last_obs)))
    return fail(MPE_EINVAL, "mpe_rollout: float outputs must be 16-byte aligned");
  if (uint64_t(e->abs_step) + uint64_t(T) > 0xFFFFFFFFull)
    return fail(MPE_EINVAL, "mpe_rollout: absolute step counter would overflow 32 bits");
  const RolloutArgs A = rollout_args(e, T, obs_traj, act_traj, rew_traj, done_traj, last_obs);
  if (e->has_gru) {
    TagArgs TA{};
    TA.r = A;
    TA.tg = e->tg;
    TA.actions_in = nullptr;
    const char* why = nullptr;
    hipError_t err = launch_rollout_gru(e->tag, e->N, e->L, e->G, TA, e->gru, nullptr, e->hidden,
                                        static_cast<hipStream_t>(stream), &why);
    if (why) return fail(MPE_EINVAL, "mpe_rollout: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout: %s", hipGetErrorString(err));
  } else if (e->tag) {
    TagArgs TA{};
    TA.r = A;
    TA.tg = e->tg;
    TA.actions_in = nullptr;
    const char* why = nullptr;
    const int mode = !e->has_policy ? 1 : (e->cfg.weight_dtype == MPE_WEIGHTS_BF16 ? 3 : 2);
    hipError_t err = launch_tag_rollout(e->N, e->L, e->G, mode, TA, e->pol.packed, nullptr,
                                        static_cast<hipStream_t>(stream), &why);
    if (why) return fail(MPE_EINVAL, "mpe_rollout: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout: %s", hipGetErrorString(err));
  } else if (e->has_policy) {
    const char* why = nullptr;
    hipError_t err = launch_rollout_policy(e->N, e->H, e->cfg.weight_dtype, A, e->pol,
                                           static_cast<hipStream_t>(stream), &why);
    if (why) return fail(MPE_EINVAL, "mpe_rollout: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout: %s", hipGetErrorString(err));
  } else {
    launch_rollout_uniform(e->N, A, static_cast<hipStream_t>(stream));
  }
  MPE_HIP(hipGetLastError());
  e->abs_step += uint32_t(T);
  return MPE_OK;
}

int mpe_set_gru_policy(mpe_env* e, const float* We, const float* be, const float* Wi, const float* bi,
                       const float* Wh, const float* bh, const float* Wf, const float* bf, const float* Wo,
                       const float* bo, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_gru_policy: NULL handle");
  int given = 0;
  for (const float* p : {We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo}) given += p != nullptr;
  if (given == 0) {
    e->has_gru = false;
    return MPE_OK;
  }
  if (given != 10) return fail(MPE_EINVAL, "mpe_set_gru_policy: pass all ten arrays or none");
  if (!gru_supported(e->tag, e->N, e->L, e->G, e->H, e->cfg.weight_dtype))
    return fail(MPE_EINVAL, "mpe_set_gru_policy: the recurrent policy needs hidden 128 and MPE_WEIGHTS_BF16 (simple "
                            "spread: 1..10 agents; predator-prey: every shape mpe_create accepts)");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!e->hidden) {
    const size_t n = size_t(e->TE) * e->N * 128;
    MPE_HIP(hipMalloc(&e->hidden, n * sizeof(float)));
    launch_fill_zero(e->hidden, n, s);
    MPE_HIP(hipGetLastError());
  }
  // until the new image is packed the handle has no recurrent policy: a failure below must not leave an
  // earlier one installed on a partly rewritten buffer
  e->has_gru = false;
  hipError_t err = pack_policy_gru(e->gru, e->D, int(e->R), We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo, s);
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_set_gru_policy: %s", hipGetErrorString(err));
  e->has_gru = true;
  return MPE_OK;
}

int mpe_set_gru_critic(mpe_env* e, const float* Wc, const float* bc, const float* wv, const float* bv, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_gru_critic: NULL handle");
  const int given = (Wc != nullptr) + (bc != nullptr) + (wv != nullptr) + (bv != nullptr);
  if (given == 0) {
    e->has_gru_critic = false;
    return MPE_OK;
  }
  if (given != 4) return fail(MPE_EINVAL, "mpe_set_gru_critic: pass all four arrays or none");
  if (!gru_supported(e->tag, e->N, e->L, e->G, e->H, e->cfg.weight_dtype))
    return fail(MPE_EINVAL, "mpe_set_gru_critic: the recurrent actor-critic needs hidden 128 and MPE_WEIGHTS_BF16");
  e->has_gru_critic = false;   // as in mpe_set_gru_policy
  hipError_t err = pack_gru_critic(e->gru_critic, int(e->R), Wc, bc, wv, bv, static_cast<hipStream_t>(stream));
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_set_gru_critic: %s", hipGetErrorString(err));
  e->has_gru_critic = true;
  return MPE_OK;
}

int mpe_get_hidden(mpe_env* e, float* hidden, void* stream) {
  if (!e || !hidden) return fail(MPE_EINVAL, "mpe_get_hidden: NULL argument");
  if (!e->hidden) return fail(MPE_ESTATE, "mpe_get_hidden: no recurrent policy has been set");
  MPE_HIP(hipMemcpyAsync(hidden, e->hidden, size_t(e->TE) * e->N * 128 * sizeof(float), hipMemcpyDeviceToDevice,
                         static_cast<hipStream_t>(stream)));
  return MPE_OK;
}

int mpe_set_hidden(mpe_env* e, const float* hidden, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_hidden: NULL handle");
  if (!e->hidden) return fail(MPE_ESTATE, "mpe_set_hidden: no recurrent policy has been set");
  const size_t n = size_t(e->TE) * e->N * 128;
  if (hidden) {
    MPE_HIP(hipMemcpyAsync(e->hidden, hidden, n * sizeof(float), hipMemcpyDeviceToDevice,
                           static_cast<hipStream_t>(stream)));
  } else {
    launch_fill_zero(e->hidden, n, static_cast<hipStream_t>(stream));
    MPE_HIP(hipGetLastError());
  }
  return MPE_OK;
}

int mpe_set_barrier_poll_limit(mpe_env* e, uint32_t polls) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_barrier_poll_limit: NULL handle");
  e->barrier_polls = polls == 0u ? (1u << 24) : polls;
  return MPE_OK;
}

int mpe_set_critic(mpe_env* e, const float* V1, const float* c1, const float* V2, const float* c2,
                   const float* V3, const float* c3, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_critic: NULL handle");
  const int given = (V1 != nullptr) + (c1 != nullptr) + (V2 != nullptr) + (c2 != nullptr) +
                    (V3 != nullptr) + (c3 != nullptr);
  if (given == 0) {
    e->has_critic = false;
    return MPE_OK;
  }
  if (given != 6) return fail(MPE_EINVAL, "mpe_set_critic: pass all six arrays or none");
  hipError_t err;
  e->has_critic = false;   // as in mpe_set_policy
  if (e->tag) {
    if (!tag_policy_supported(e->N, e->L, e->G, e->H, e->cfg.weight_dtype))
      return fail(MPE_EINVAL, "mpe_set_critic: unsupported shape: the MPE_SCENARIO_TAG actor-critic rollout is built "
                              "for hidden 64 and observation rows of at most 32 floats");
    err = pack_policy_tag(e->critic, e->N, e->L, e->G, int(e->R), e->cfg.weight_dtype == MPE_WEIGHTS_BF16, 1, V1, c1,
                          V2, c2, V3, c3, static_cast<hipStream_t>(stream));
  } else if (e->cfg.weight_dtype == MPE_WEIGHTS_BF16 && wide_supported(e->N, e->H)) {
    err = pack_policy_wide(e->critic, e->N, e->H, int(e->R), V1, c1, V2, c2, V3, c3, 1, static_cast<hipStream_t>(stream));
  } else {
    if (!f32_supported(e->N, e->H, e->cfg.weight_dtype == MPE_WEIGHTS_BF16))
      return fail(MPE_EINVAL, "mpe_set_critic: unsupported shape: the actor-critic rollout is built for the "
                              "shapes of mpe_set_policy");
    err = pack_policy_f32(e->critic, e->N, int(e->R), V1, c1, V2, c2, V3, c3, 1,
                          e->cfg.weight_dtype == MPE_WEIGHTS_BF16, static_cast<hipStream_t>(stream));
  }
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_set_critic: %s", hipGetErrorString(err));
  e->has_critic = true;
  return MPE_OK;
}

int mpe_rollout_ac(mpe_env* e, int32_t T, float* obs_traj, uint8_t* act_traj, float* logp_traj,
                   float* value_traj, float* rew_traj, uint8_t* done_traj, float* last_obs,
                   float* last_value, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_rollout_ac: NULL handle");
  if (T < 1 || T > MPE_MAX_ROLLOUT_STEPS)
    return fail(MPE_EINVAL, "mpe_rollout_ac: T must be in [1, %d] (got %d)", MPE_MAX_ROLLOUT_STEPS, T);
  if (!e->ready) return fail(MPE_ESTATE, "mpe_rollout_ac: call mpe_reset or mpe_set_state first");
  if (int rc = check_fault(e, "mpe_rollout_ac")) return rc;
  if (e->has_gru) {
    if (!e->has_gru_critic)
      return fail(MPE_ESTATE, "mpe_rollout_ac: with a recurrent policy, needs mpe_set_gru_critic first");
  } else if (!e->has_policy || !e->has_critic) {
    return fail(MPE_ESTATE, "mpe_rollout_ac: needs mpe_set_policy and mpe_set_critic (or mpe_set_gru_policy and "
                            "mpe_set_gru_critic) first");
  }
  const bool wide = !e->tag && e->cfg.weight_dtype == MPE_WEIGHTS_BF16 && wide_supported(e->N, e->H);
  if (!e->has_gru && !e->tag && !wide && !f32_supported(e->N, e->H, e->cfg.weight_dtype == MPE_WEIGHTS_BF16))
    return fail(MPE_EINVAL, "mpe_rollout_ac: unsupported shape");
  for (const float* p : {obs_traj, logp_traj, value_traj, rew_traj, last_obs, last_value})
    if (p && !aligned16(p)) return fail(MPE_EINVAL, "mpe_rollout_ac: float outputs must be 16-byte aligned");
  if (uint64_t(e->abs_step) + uint64_t(T) > 0xFFFFFFFFull)
    return fail(MPE_EINVAL, "mpe_rollout_ac: absolute step counter would overflow 32 bits");
  RolloutArgs A = rollout_args(e, T, obs_traj, act_traj, rew_traj, done_traj, last_obs);
  A.logp_traj = logp_traj;
  A.value_traj = value_traj;
  A.last_value = last_value;
  const char* why = nullptr;
  hipError_t err;
  if (e->has_gru) {
    TagArgs TA{};
    TA.r = A;
    TA.tg = e->tg;
    TA.actions_in = nullptr;
    err = launch_rollout_gru(e->tag, e->N, e->L, e->G, TA, e->gru, e->gru_critic.packed, e->hidden,
                             static_cast<hipStream_t>(stream), &why);
  } else if (e->tag) {
    TagArgs TA{};
    TA.r = A;
    TA.tg = e->tg;
    TA.actions_in = nullptr;
    err = launch_tag_rollout(e->N, e->L, e->G, e->cfg.weight_dtype == MPE_WEIGHTS_BF16 ? 5 : 4, TA, e->pol.packed,
                             e->critic.packed, static_cast<hipStream_t>(stream), &why);
  } else if (wide) {
    err = launch_rollout_ac_wide(e->N, e->H, A, e->pol, e->critic, static_cast<hipStream_t>(stream), &why);
  } else {
    err = launch_rollout_ac_f32(e->N, e->cfg.weight_dtype == MPE_WEIGHTS_BF16, A, e->pol, e->critic,
                                static_cast<hipStream_t>(stream), &why);
  }
  if (why) return fail(MPE_EINVAL, "mpe_rollout_ac: %s", why);
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout_ac: %s", hipGetErrorString(err));
  MPE_HIP(hipGetLastError());
  e->abs_step += uint32_t(T);
  return MPE_OK;
}

int mpe_get_state(mpe_env* e, float* pos_a, float* vel_a, float* pos_l, int32_t* ep_step,
                  uint32_t* abs_step, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_get_state: NULL handle");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t nf = agent_floats(e) * sizeof(float);
  if (pos_a) MPE_HIP(hipMemcpyAsync(pos_a, e->st.pos_a, nf, hipMemcpyDeviceToDevice, s));
  if (vel_a) MPE_HIP(hipMemcpyAsync(vel_a, e->st.vel_a, nf, hipMemcpyDeviceToDevice, s));
  const size_t nl = landmark_floats(e) * sizeof(float);
  if (pos_l && nl) MPE_HIP(hipMemcpyAsync(pos_l, e->st.pos_l, nl, hipMemcpyDeviceToDevice, s));
  if (ep_step)
    MPE_HIP(hipMemcpyAsync(ep_step, e->st.ep_step, size_t(e->TE) * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  if (abs_step) *abs_step = e->abs_step;
  return MPE_OK;
}

int mpe_set_state(mpe_env* e, const float* pos_a, const float* vel_a, const float* pos_l,
                  const int32_t* ep_step, uint32_t seed, uint32_t abs_step, void* stream) {
  if (!e) return fail(MPE_EINVAL, "mpe_set_state: NULL handle");
  if (!pos_a || !vel_a || (!pos_l && e->L > 0) || !ep_step) return fail(MPE_EINVAL, "mpe_set_state: NULL array");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t nf = agent_floats(e) * sizeof(float);
  MPE_HIP(hipMemcpyAsync(e->st.pos_a, pos_a, nf, hipMemcpyDeviceToDevice, s));
  MPE_HIP(hipMemcpyAsync(e->st.vel_a, vel_a, nf, hipMemcpyDeviceToDevice, s));
  const size_t nl = landmark_floats(e) * sizeof(float);
  if (nl) MPE_HIP(hipMemcpyAsync(e->st.pos_l, pos_l, nl, hipMemcpyDeviceToDevice, s));
  MPE_HIP(hipMemcpyAsync(e->st.ep_step, ep_step, size_t(e->TE) * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  e->seed = seed;
  e->abs_step = abs_step;
  e->ready = true;
  return MPE_OK;
}

// ---------------------------------------------------------------------------------------------------
// mpe_rollout_noalloc: reset + policy + T fused steps in one call that allocates nothing.  What the
// handle-based path keeps in memory of its own -- the SoA state of the environments, the packed policy
// image, the fault word -- lives in one static device array.
// ---------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[MPE_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, once known

// `scratch` in host code is only a stand-in for the symbol; the device address of this device's copy comes
// from the runtime, once per device (with that device current), and is what kernels and copies are given.
int scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout_noalloc: hipGetDevice: %s", hipGetErrorString(err));
  if (dev < 0 || dev >= kMaxDevices) return fail(MPE_EHIP, "mpe_rollout_noalloc: device ordinal %d not supported", dev);
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    err = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !sym)
      return fail(MPE_EHIP, "mpe_rollout_noalloc: hipGetSymbolAddress(scratch): %s", hipGetErrorString(err));
    p = static_cast<unsigned char*>(sym);
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return MPE_OK;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int mpe_rollout_noalloc(const mpe_config* cfg, uint32_t seed, const float* W1, const float* b1, const float* W2,
                        const float* b2, const float* W3, const float* b3, int32_t T, float* obs_traj,
                        uint8_t* act_traj, float* rew_traj, uint8_t* done_traj, float* last_obs, void* stream) {
  if (!cfg) return fail(MPE_EINVAL, "mpe_rollout_noalloc: NULL config");
  if (int rc = validate(cfg)) return rc;
  if (cfg->scenario != MPE_SCENARIO_SPREAD)
    return fail(MPE_EINVAL, "mpe_rollout_noalloc: built for MPE_SCENARIO_SPREAD");
  if (T < 1 || T > MPE_MAX_ROLLOUT_STEPS)
    return fail(MPE_EINVAL, "mpe_rollout_noalloc: T must be in [1, %d] (got %d)", MPE_MAX_ROLLOUT_STEPS, T);
  if ((obs_traj && !aligned16(obs_traj)) || (rew_traj && !aligned16(rew_traj)) || (last_obs && !aligned16(last_obs)))
    return fail(MPE_EINVAL, "mpe_rollout_noalloc: float outputs must be 16-byte aligned");
  const int given = (W1 != nullptr) + (b1 != nullptr) + (W2 != nullptr) + (b2 != nullptr) + (W3 != nullptr) + (b3 != nullptr);
  if (given != 0 && given != 6) return fail(MPE_EINVAL, "mpe_rollout_noalloc: pass all six weight arrays or none");
  mpe_env e;   // host fields only, on the stack: nothing here owns memory
  init_from_config(&e, cfg);
  size_t packed_bytes = 0;
  if (given) {
    if (e.H != 64 && e.H != 128) return fail(MPE_EINVAL, "mpe_rollout_noalloc: config.hidden must be 64 or 128");
    packed_bytes = packed_policy_bytes(e.N, e.H, int(e.R), cfg->weight_dtype);
    if (!packed_bytes)
      return fail(MPE_EINVAL, "mpe_rollout_noalloc: unsupported policy shape (see mpe_set_policy)");
  }
  // ---- layout inside the scratch array: fault word | pos_a | vel_a | pos_l | ep_step | packed policy
  const size_t nf = agent_floats(&e) * sizeof(float);
  const size_t off_pos = 256;
  const size_t off_vel = align_up(off_pos + nf, 256);
  const size_t off_lm = align_up(off_vel + nf, 256);
  const size_t off_ep = align_up(off_lm + landmark_floats(&e) * sizeof(float) + 16, 256);
  const size_t off_pk = align_up(off_ep + size_t(e.TE) * sizeof(int32_t), 256);
  const size_t need = off_pk + packed_bytes;
  if (need > size_t(MPE_NOALLOC_SCRATCH_BYTES))
    return fail(MPE_EINVAL, "mpe_rollout_noalloc: %zu envs of %d agents (and the packed policy) need %zu bytes of "
                            "library memory; the static scratch holds %zu", size_t(e.TE), e.N, need,
                size_t(MPE_NOALLOC_SCRATCH_BYTES));
  unsigned char* base = nullptr;
  if (int rc = scratch_of_current_device(&base)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  e.st.pos_a = reinterpret_cast<float*>(base + off_pos);
  e.st.vel_a = reinterpret_cast<float*>(base + off_vel);
  e.st.pos_l = reinterpret_cast<float*>(base + off_lm);
  e.st.ep_step = reinterpret_cast<int32_t*>(base + off_ep);
  e.fault_dev = reinterpret_cast<uint32_t*>(base);
  // The array keeps the last call's contents.  Cleared here: the fault word (a fill kernel, not a memset node, so
  // that the call can be captured into a graph).  Overwritten in full before use: the state (reset kernel) and
  // the packed image (the pack kernel writes every byte of it that a rollout kernel reads).
  launch_fill_zero(reinterpret_cast<float*>(base), 1, s);
  launch_reset(e.N, e.st, e.TE, e.E, seed, nullptr, s);
  MPE_HIP(hipGetLastError());
  e.seed = seed;
  e.abs_step = 0;
  const RolloutArgs A = rollout_args(&e, T, obs_traj, act_traj, rew_traj, done_traj, last_obs);
  const char* why = nullptr;
  if (given) {
    e.pol.packed = base + off_pk;
    e.pol.bytes = packed_bytes;
    e.pol.borrowed = true;
    hipError_t err = pack_policy(e.pol, e.N, e.H, int(e.R), cfg->weight_dtype, W1, b1, W2, b2, W3, b3, s, &why);
    if (why) return fail(MPE_EINVAL, "mpe_rollout_noalloc: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout_noalloc: %s", hipGetErrorString(err));
    err = launch_rollout_policy(e.N, e.H, cfg->weight_dtype, A, e.pol, s, &why);
    if (why) return fail(MPE_EINVAL, "mpe_rollout_noalloc: %s", why);
    if (err != hipSuccess) return fail(MPE_EHIP, "mpe_rollout_noalloc: %s", hipGetErrorString(err));
  } else {
    launch_rollout_uniform(e.N, A, s);
  }
  MPE_HIP(hipGetLastError());
  return MPE_OK;
}

}  // extern "C"
