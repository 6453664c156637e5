// Environment-only kernels: reset, single step, and the persistent T-step rollout with
// seeded uniform actions.  One lane owns one environment; the whole state of that env stays
// in registers for the T steps of a rollout and only the trajectory leaves the chip.
#include "mpe_launch.h"

namespace mpe {

namespace {

struct Lane {
  size_t g;       // global env index
  uint32_t run;   // g / E
  uint32_t env;   // g % E
  bool valid;
  size_t g0;      // first env of this wave
  int nvalid;     // number of valid envs in this wave
  int lane;
};

__device__ __forceinline__ Lane lane_info(uint32_t TE, uint32_t E) {
  Lane L;
  L.lane = threadIdx.x;
  L.g0 = size_t(blockIdx.x) * kWave;
  L.g = L.g0 + L.lane;
  L.valid = L.g < TE;
  const uint32_t gc = L.valid ? uint32_t(L.g) : 0u;
  L.run = gc / E;
  L.env = gc - L.run * E;
  const size_t left = size_t(TE) - L.g0;
  L.nvalid = left < size_t(kWave) ? int(left) : kWave;
  return L;
}

template <int N>
__global__ __launch_bounds__(kWave) void reset_kernel(StatePtrs st, uint32_t TE, uint32_t E,
                                                      uint32_t seed, float* __restrict__ obs) {
  __shared__ __attribute__((aligned(16))) float tile[ObsTile<N>::kFloats];
  const Lane L = lane_info(TE, E);
  Env<N> s;
  reset_env<N>(s, seed, L.run, L.env, 0u);
  if (L.valid) store_state<N>(s, st, TE, L.g);
  if (obs) emit_obs<N>(s, tile, obs, L.g0, L.nvalid, L.lane);
}

template <int N>
__global__ __launch_bounds__(kWave) void step_kernel(StatePtrs st, Phys ph, uint32_t TE, uint32_t E,
                                                     uint32_t seed, uint32_t abs_step,
                                                     const uint8_t* __restrict__ actions,
                                                     float* __restrict__ obs, float* __restrict__ reward,
                                                     uint8_t* __restrict__ done) {
  __shared__ __attribute__((aligned(16))) float tile[ObsTile<N>::kFloats];
  const Lane L = lane_info(TE, E);
  Env<N> s;
  uint32_t a[N];
  if (L.valid) {
    load_state<N>(s, st, TE, L.g);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint32_t v = actions[L.g * N + i];
      a[i] = v < uint32_t(kNumActions) ? v : 0u;
    }
  } else {
    zero_env<N>(s);
#pragma unroll
    for (int i = 0; i < N; ++i) a[i] = 0u;
  }
  float r;
  bool d;
  transition<N>(s, a, ph, seed, L.run, L.env, abs_step, r, d);
  if (L.valid) {
    store_state<N>(s, st, TE, L.g);
    if (reward) reward[L.g] = r;
    if (done) done[L.g] = d ? 1 : 0;
  }
  if (obs) emit_obs<N>(s, tile, obs, L.g0, L.nvalid, L.lane);
}

// Persistent rollout with uniform random actions (no policy installed).
template <int N>
__global__ __launch_bounds__(kWave) void rollout_uniform_kernel(RolloutArgs A) {
  __shared__ __attribute__((aligned(16))) float tile[ObsTile<N>::kFloats];
  constexpr int D = 6 * N;
  const Lane L = lane_info(A.TE, A.E);
  Env<N> s;
  if (L.valid) load_state<N>(s, A.st, A.TE, L.g); else zero_env<N>(s);
  const size_t TE = A.TE;
  for (int t = 0; t < A.T; ++t) {
    const uint32_t step = A.abs_step + uint32_t(t);
    if (A.obs_traj) emit_obs<N>(s, tile, A.obs_traj + size_t(t) * TE * N * D, L.g0, L.nvalid, L.lane);
    uint32_t a[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint4 w = philox4x32_10(L.env, step, uint32_t(i), kTagUniformAction, A.seed, L.run);
      a[i] = word_to_action(w.x);
    }
    if (A.act_traj && L.valid) {
      uint8_t* dst = A.act_traj + (size_t(t) * TE + L.g) * N;
#pragma unroll
      for (int i = 0; i < N; ++i) dst[i] = uint8_t(a[i]);
    }
    float r;
    bool d;
    transition<N>(s, a, A.ph, A.seed, L.run, L.env, step, r, d);
    if (L.valid) {
      if (A.rew_traj) A.rew_traj[size_t(t) * TE + L.g] = r;
      if (A.done_traj) A.done_traj[size_t(t) * TE + L.g] = d ? 1 : 0;
    }
  }
  if (A.last_obs) emit_obs<N>(s, tile, A.last_obs, L.g0, L.nvalid, L.lane);
  if (L.valid) store_state<N>(s, A.st, A.TE, L.g);
}

inline dim3 env_grid(uint32_t TE) { return dim3((TE + kWave - 1) / kWave); }

template <int N>
struct EnvLaunch {
  static void reset(const StatePtrs& st, uint32_t TE, uint32_t E, uint32_t seed, float* obs, hipStream_t s) {
    hipLaunchKernelGGL(reset_kernel<N>, env_grid(TE), dim3(kWave), 0, s, st, TE, E, seed, obs);
  }
  static void step(const StatePtrs& st, const Phys& ph, uint32_t TE, uint32_t E, uint32_t seed,
                   uint32_t abs_step, const uint8_t* actions, float* obs, float* reward, uint8_t* done,
                   hipStream_t s) {
    hipLaunchKernelGGL(step_kernel<N>, env_grid(TE), dim3(kWave), 0, s, st, ph, TE, E, seed, abs_step,
                       actions, obs, reward, done);
  }
  static void rollout(const RolloutArgs& A, hipStream_t s) {
    hipLaunchKernelGGL(rollout_uniform_kernel<N>, env_grid(A.TE), dim3(kWave), 0, s, A);
  }
};

}  // namespace

#define MPE_DISPATCH_N(N_, CALL)                 \
  switch (N_) {                                  \
    case 1: { constexpr int kN = 1; CALL; } break;   \
    case 2: { constexpr int kN = 2; CALL; } break;   \
    case 3: { constexpr int kN = 3; CALL; } break;   \
    case 4: { constexpr int kN = 4; CALL; } break;   \
    case 5: { constexpr int kN = 5; CALL; } break;   \
    case 6: { constexpr int kN = 6; CALL; } break;   \
    case 7: { constexpr int kN = 7; CALL; } break;   \
    case 8: { constexpr int kN = 8; CALL; } break;   \
    case 9: { constexpr int kN = 9; CALL; } break;   \
    case 10: { constexpr int kN = 10; CALL; } break; \
    default: break;                              \
  }

void launch_reset(int N, const StatePtrs& st, uint32_t TE, uint32_t E, uint32_t seed, float* obs,
                  hipStream_t s) {
  MPE_DISPATCH_N(N, EnvLaunch<kN>::reset(st, TE, E, seed, obs, s));
}

void launch_step(int N, const StatePtrs& st, const Phys& ph, uint32_t TE, uint32_t E, uint32_t seed,
                 uint32_t abs_step, const uint8_t* actions, float* obs, float* reward, uint8_t* done,
                 hipStream_t s) {
  MPE_DISPATCH_N(N, EnvLaunch<kN>::step(st, ph, TE, E, seed, abs_step, actions, obs, reward, done, s));
}

void launch_rollout_uniform(int N, const RolloutArgs& A, hipStream_t s) {
  MPE_DISPATCH_N(N, EnvLaunch<kN>::rollout(A, s));
}

}  // namespace mpe
