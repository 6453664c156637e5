// Host-side launch interface between the C ABI (mpe_api.hip) and the kernel files.
#pragma once

#include <atomic>

#include "mpe_device.h"

namespace mpe {

// A kernel that needs more than 64 KB of dynamic LDS must be allowed to, once per device it is
// launched on (function attributes belong to the device's copy of the code).  `done` holds one bit
// per device ordinal; setting the attribute twice from two threads is harmless.
inline hipError_t allow_lds(const void* kern, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (unsigned(dev) & 63u);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes));
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Compute units of the current device (queried once per process; launch shapes are chosen by it).
inline uint32_t compute_units() {
  static std::atomic<int> cus{0};
  int n = cus.load(std::memory_order_relaxed);
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cus.store(n, std::memory_order_relaxed);
  }
  return uint32_t(n);
}

struct RolloutArgs {
  StatePtrs st;
  Phys ph;
  uint32_t TE;        // total envs = runs * envs per run
  uint32_t E;         // envs per run
  uint32_t seed;
  uint32_t abs_step;  // absolute step of the first transition
  int32_t T;
  float* obs_traj;    // [T][TE][N][D] or null
  uint8_t* act_traj;  // [T][TE][N]    or null
  float* rew_traj;    // [T][TE]       or null
  uint8_t* done_traj; // [T][TE]       or null
  float* last_obs;    // [TE][N][D]    or null
  // actor-critic rollout only (null otherwise)
  float* logp_traj = nullptr;   // [T][TE][N] log-probability of the sampled action
  float* value_traj = nullptr;  // [T][TE][N] critic value of the observation acted on
  float* last_value = nullptr;  // [TE][N]    critic value of last_obs
  // Word that a kernel raises (system scope) when a bounded wait gave up; null = not reported.
  uint32_t* fault = nullptr;
  // Polls after which a wait at a sync-group barrier gives up (kBarrierSpinLimit unless a test lowers it).
  uint32_t barrier_polls = 1u << 24;
};

// Predator-prey scenario: constants by role (index 0 adversary, 1 good agent), combined on the
// host in double and rounded once.
struct TagPhys {
  float dt, keep, dt_over_mass, inv_margin, force_margin;
  int32_t max_ep;
  float radius[2];
  float gain[2];
  float limit[2];      // speed limit
  float limit_sq[2];
  float lm_radius;
  float touch_sq;      // (adversary radius + good radius)^2
};

struct TagArgs {
  RolloutArgs r;                 // state, sizes, seed, step, outputs (r.ph is unused)
  TagPhys tg;
  const uint8_t* actions_in;     // [TE][N], single step with given actions only
};

// (N, L, G) = agents, landmarks, good agents
bool tag_supported(int N, int L, int G);
bool tag_policy_supported(int N, int L, int G, int H, int weight_dtype);
void launch_tag_reset(int N, int L, int G, const StatePtrs& st, uint32_t TE, uint32_t E, uint32_t seed, float* obs,
                      hipStream_t s);
// mode 0: one step under A.actions_in (r.T must be 1; obs after the step -> r.last_obs, reward ->
// r.rew_traj, done -> r.done_traj); mode 1: uniform random actions; mode 2: the packed fp32 policy;
// mode 3: the packed bf16 policy; mode 4 / 5: the packed fp32 / bf16 policy and critic (actor-critic outputs in r)
hipError_t launch_tag_rollout(int N, int L, int G, int mode, const TagArgs& A, const void* packed,
                              const void* packed_critic, hipStream_t s, const char** why);
struct PolicyBuffers;
// nout: outputs of the last layer (5 policy logits, 1 critic value)
hipError_t pack_policy_tag(PolicyBuffers& pb, int N, int L, int G, int R, bool bf16, int nout, const float* W1,
                           const float* b1, const float* W2, const float* b2, const float* W3, const float* b3,
                           hipStream_t s);

void launch_reset(int N, const StatePtrs& st, uint32_t TE, uint32_t E, uint32_t seed, float* obs,
                  hipStream_t s);
void launch_step(int N, const StatePtrs& st, const Phys& ph, uint32_t TE, uint32_t E, uint32_t seed,
                 uint32_t abs_step, const uint8_t* actions, float* obs, float* reward, uint8_t* done,
                 hipStream_t s);
void launch_rollout_uniform(int N, const RolloutArgs& A, hipStream_t s);

// Policy weights re-packed into MFMA A-operand order (device memory owned by the handle, or, `borrowed`,
// a piece of memory of `bytes` bytes that is never freed or grown here).
struct PolicyBuffers {
  void* packed = nullptr;
  size_t bytes = 0;
  bool borrowed = false;
};
// Bytes that pack_policy writes for R runs (0 for an unsupported shape).
size_t packed_policy_bytes(int N, int H, int R, int weight_dtype);

// Both return a HIP status; *why is set (and nothing launched) when the shape is unsupported.
hipError_t pack_policy(PolicyBuffers& pb, int N, int H, int R, int weight_dtype, const float* W1,
                       const float* b1, const float* W2, const float* b2, const float* W3,
                       const float* b3, hipStream_t s, const char** why);
hipError_t launch_rollout_policy(int N, int H, int weight_dtype, const RolloutArgs& A,
                                 const PolicyBuffers& pb, hipStream_t s, const char** why);
void free_policy(PolicyBuffers& pb);

// Per-kernel-family entry points behind pack_policy / launch_rollout_policy.
bool wide_supported(int N, int H);                       // bf16 general kernel
size_t packed_run_bytes_wide(int N, int H);
hipError_t pack_policy_wide(PolicyBuffers& pb, int N, int H, int R, const float* W1, const float* b1,
                            const float* W2, const float* b2, const float* W3, const float* b3, int nout,
                            hipStream_t s);
hipError_t launch_rollout_ac_wide(int N, int H, const RolloutArgs& A, const PolicyBuffers& pb,
                                  const PolicyBuffers& critic, hipStream_t s, const char** why);
hipError_t launch_rollout_policy_wide(int N, int H, const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s,
                                      const char** why);
bool uniform_wide_supported(int N);                      // env-only rollout with the wide kernel's mapping
hipError_t launch_rollout_uniform_wide(int N, const RolloutArgs& A, hipStream_t s);
bool f32_supported(int N, int H, bool bf16);             // headline kernel (H = 64; N <= 3, with fp32 weights N <= 10)
size_t packed_run_bytes_f32(int N, bool bf16);
hipError_t pack_policy_f32(PolicyBuffers& pb, int N, int R, const float* W1, const float* b1, const float* W2,
                           const float* b2, const float* W3, const float* b3, int nout, bool bf16, hipStream_t s);
hipError_t launch_rollout_ac_f32(int N, bool bf16, const RolloutArgs& A, const PolicyBuffers& pb,
                                 const PolicyBuffers& critic, hipStream_t s, const char** why);
hipError_t launch_rollout_policy_f32(int N, bool bf16, const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s,
                                     const char** why);
hipError_t ensure_policy_bytes(PolicyBuffers& pb, size_t bytes);

// Recurrent policy (hidden 128, bf16): simple spread with 1..3 agents.
// tag: the predator-prey scenario with (N, L, G) agents, landmarks, good agents; otherwise simple spread (L, G unused)
bool gru_supported(bool tag, int N, int L, int G, int H, int weight_dtype);
// D = observation width of the scenario
hipError_t pack_policy_gru(PolicyBuffers& pb, int D, int R, const float* We, const float* be, const float* Wi,
                           const float* bi, const float* Wh, const float* bh, const float* Wf, const float* bf,
                           const float* Wo, const float* bo, hipStream_t s);
// hidden: [TE][N][128] fp32, read at the start and written at the end of the rollout; A.tg is read by the
// predator-prey shapes only
// critic: the packed critic head (pack_gru_critic) for the actor-critic rollout (A.r.logp_traj, value_traj,
// last_value), or null for the plain one
hipError_t launch_rollout_gru(bool tag, int N, int L, int G, const TagArgs& A, const PolicyBuffers& pb, const void* critic,
                              float* hidden, hipStream_t s, const char** why);
// Critic head of the recurrent actor-critic: Wc [R][128][128], bc [R][128], wv [R][128], bv [R]
hipError_t pack_gru_critic(PolicyBuffers& pb, int R, const float* Wc, const float* bc, const float* wv, const float* bv,
                           hipStream_t s);
void launch_fill_zero(float* p, size_t n, hipStream_t s);

}  // namespace mpe
