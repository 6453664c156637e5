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
  if (obs) emit_obs<N>(s, tile, obs + L.g0 * (N * 6 * N), L.nvalid, L.lane);
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
  bool d;
  if (ph.reward_mode == 1) {
    float r[N];
    transition<N, true>(s, a, ph, seed, L.run, L.env, abs_step, r, d);
    if (L.valid && reward) {
#pragma unroll
      for (int i = 0; i < N; ++i) reward[L.g * N + i] = r[i];
    }
  } else {
    float r[1];
    transition<N>(s, a, ph, seed, L.run, L.env, abs_step, r, d);
    if (L.valid && reward) reward[L.g] = r[0];
  }
  if (L.valid) {
    store_state<N>(s, st, TE, L.g);
    if (done) done[L.g] = d ? 1 : 0;
  }
  if (obs) emit_obs<N>(s, tile, obs + L.g0 * (N * 6 * N), L.nvalid, L.lane);
}

// Persistent rollout with uniform random actions (no policy installed).  Output pointers are
// advanced by one time slice per step instead of being recomputed from (t, env).  PER_AGENT:
// rew_traj is [T][TE][N] (mixed per-agent reward).
template <int N, bool PER_AGENT>
__global__ __launch_bounds__(kWave) void rollout_uniform_kernel(RolloutArgs A) {
  __shared__ __attribute__((aligned(16))) float tile[ObsTile<N>::kFloats];
  constexpr int D = 6 * N;
  const Lane L = lane_info(A.TE, A.E);
  Env<N> s;
  if (L.valid) load_state<N>(s, A.st, A.TE, L.g); else zero_env<N>(s);
  const size_t TE = A.TE;
  float* obs_p = A.obs_traj ? A.obs_traj + L.g0 * (N * D) : nullptr;
  uint8_t* act_p = (A.act_traj && L.valid) ? A.act_traj + L.g * N : nullptr;
  constexpr int RW = PER_AGENT ? N : 1;   // rewards per env and step
  float* rew_p = (A.rew_traj && L.valid) ? A.rew_traj + L.g * RW : nullptr;
  uint8_t* done_p = (A.done_traj && L.valid) ? A.done_traj + L.g : nullptr;
  uint32_t step = A.abs_step;
  for (int t = 0; t < A.T; ++t, ++step) {
    if (obs_p) {
      emit_obs<N>(s, tile, obs_p, L.nvalid, L.lane);
      obs_p += TE * (N * D);
    }
    uint32_t a[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint4 w = philox4x32_10(L.env, step, uint32_t(i), kTagUniformAction, A.seed, L.run);
      a[i] = word_to_action(w.x);
    }
    if (act_p) {
#pragma unroll
      for (int i = 0; i < N; ++i) act_p[i] = uint8_t(a[i]);
      act_p += TE * N;
    }
    float r[RW];
    bool d;
    transition<N, PER_AGENT>(s, a, A.ph, A.seed, L.run, L.env, step, r, d);
    if (rew_p) {
#pragma unroll
      for (int i = 0; i < RW; ++i) rew_p[i] = r[i];
      rew_p += TE * RW;
    }
    if (done_p) { *done_p = d ? 1 : 0; done_p += TE; }
  }
  if (A.last_obs) emit_obs<N>(s, tile, A.last_obs + L.g0 * (N * D), L.nvalid, L.lane);
  if (L.valid) store_state<N>(s, A.st, A.TE, L.g);
}

// --------------------------------------------------------------------------------------
// Wave-specialised persistent rollout for N <= 3, whole waves only (TE % 64 == 0, 16-byte
// aligned time slices).  A block is two wavefronts over the same 64 envs:
//   wave 0 (compute) keeps the 64 envs in registers, steps them, and drops each finished time
//           slice -- obs, reward, actions, done -- into one of two LDS slice buffers;
//   wave 1 (writer)  copies finished slices to HBM with 16-byte stores covering whole lines.
// The stores of a 1.9 GB trajectory back-pressure the issuing wave for most of a step; in a
// single wave that stall serialises with the arithmetic of the next step, here it overlaps.
// Two barriers per step hand the buffers back and forth:
//   X_t: writer has read slice t-1 out of buf[(t+1)&1]  -> compute may overwrite it
//   Y_t: compute has completed slice t in buf[t&1]       -> writer may read it
// Blocks are mapped to env groups XCD-aware: the hardware deals block b to XCD b % 8, so
// group = (b % 8) * groups_per_xcd + b / 8 gives each XCD one contiguous range of envs and
// the partial cache lines of neighbouring groups (actions: 192 B, done: 64 B per group and
// step) meet in the same L2 instead of being written back separately.
// --------------------------------------------------------------------------------------
template <int N>
struct SliceBuf {
  static constexpr int D = 6 * N;
  static constexpr int OBS_BYTES = kWave * N * D * 4;
  static constexpr int REW_OFF = OBS_BYTES;            // 64 floats
  static constexpr int ACT_OFF = REW_OFF + kWave * 4;  // 64 * N bytes
  static constexpr int DONE_OFF = ACT_OFF + kWave * N; // 64 bytes
  static constexpr int BYTES = (DONE_OFF + kWave + 15) & ~15;
  static constexpr int OBS_F4 = OBS_BYTES / 16;
  static constexpr int FULL = OBS_F4 / kWave;          // full 64-lane rounds of obs
  static constexpr int TAIL = OBS_F4 % kWave;          // obs float4 left for the mixed round
  static constexpr int REW_L = TAIL, ACT_L = REW_L + 16, DONE_L = ACT_L + 4 * N, END_L = DONE_L + 4;
  static_assert(END_L <= kWave, "mixed round must fit one wavefront");
};

template <int N>
__global__ __launch_bounds__(2 * kWave) void rollout_uniform_ws_kernel(RolloutArgs A, uint32_t groups,
                                                                       uint32_t groups_per_xcd) {
  using SB = SliceBuf<N>;
  constexpr int D = 6 * N;
  __shared__ __attribute__((aligned(16))) uint8_t buf[2][SB::BYTES];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t grp = (blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3);
  if (grp >= groups) return;  // whole block, before any barrier
  const size_t TE = A.TE;
  const size_t g0 = size_t(grp) * kWave;

  if (wave == 0) {
    // ------------------------------------------------------------------ compute wave
    const size_t g = g0 + lane;
    const uint32_t run = uint32_t(g) / A.E;
    const uint32_t env = uint32_t(g) - run * A.E;
    Env<N> s;
    load_state<N>(s, A.st, TE, g);
    auto write_obs = [&](uint8_t* b) {
      float2* row = reinterpret_cast<float2*>(b) + lane * (N * D / 2);
#pragma unroll
      for (int i = 0; i < N; ++i) build_agent_obs<N>(s, i, row + i * (D / 2));
    };
    write_obs(buf[0]);
    uint32_t step = A.abs_step;
    for (int t = 0; t < A.T; ++t, ++step) {
      uint32_t a[N];
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const uint4 w = philox4x32_10(env, step, uint32_t(i), kTagUniformAction, A.seed, run);
        a[i] = word_to_action(w.x);
      }
      float r[1];
      bool d;
      transition<N>(s, a, A.ph, A.seed, run, env, step, r, d);
      __syncthreads();  // X_t
      uint8_t* cur = buf[t & 1];
      reinterpret_cast<float*>(cur + SB::REW_OFF)[lane] = r[0];
#pragma unroll
      for (int i = 0; i < N; ++i) cur[SB::ACT_OFF + lane * N + i] = uint8_t(a[i]);
      cur[SB::DONE_OFF + lane] = d ? 1 : 0;
      write_obs(buf[(t + 1) & 1]);
      __syncthreads();  // Y_t
    }
    if (A.last_obs) stream_out_full<SB::OBS_F4>(reinterpret_cast<const float*>(buf[A.T & 1]),
                                                A.last_obs + g0 * (N * D), lane);
    store_state<N>(s, A.st, TE, g);
  } else {
    // ------------------------------------------------------------------ writer wave
    // Full rounds: lane l moves obs float4 number k*64 + l.  Mixed round: the obs tail, then
    // reward (16 lanes), actions (4N lanes) and done (4 lanes), one float4 each.
    uint8_t* obs_g = A.obs_traj ? reinterpret_cast<uint8_t*>(A.obs_traj + g0 * (N * D)) + lane * 16 : nullptr;
    const size_t obs_stride = TE * (N * D) * 4;
    int mix_lds = -1;          // byte offset inside a slice buffer, -1: lane idle in the mixed round
    uint8_t* mix_g = nullptr;
    size_t mix_stride = 0;
    if (lane < SB::TAIL) {
      if (A.obs_traj) {
        mix_lds = (SB::FULL * kWave + lane) * 16;
        mix_g = reinterpret_cast<uint8_t*>(A.obs_traj + g0 * (N * D)) + mix_lds;
        mix_stride = obs_stride;
      }
    } else if (lane < SB::ACT_L) {
      if (A.rew_traj) {
        mix_lds = SB::REW_OFF + (lane - SB::REW_L) * 16;
        mix_g = reinterpret_cast<uint8_t*>(A.rew_traj + g0) + (lane - SB::REW_L) * 16;
        mix_stride = TE * 4;
      }
    } else if (lane < SB::DONE_L) {
      if (A.act_traj) {
        mix_lds = SB::ACT_OFF + (lane - SB::ACT_L) * 16;
        mix_g = A.act_traj + g0 * N + (lane - SB::ACT_L) * 16;
        mix_stride = TE * N;
      }
    } else if (lane < SB::END_L) {
      if (A.done_traj) {
        mix_lds = SB::DONE_OFF + (lane - SB::DONE_L) * 16;
        mix_g = A.done_traj + g0 + (lane - SB::DONE_L) * 16;
        mix_stride = TE;
      }
    }
    v4f v[SB::FULL > 0 ? SB::FULL : 1];
    v4f vm = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int t = 0; t <= A.T; ++t) {
      if (t > 0) {
        if (obs_g) {
#pragma unroll
          for (int k = 0; k < SB::FULL; ++k) __builtin_nontemporal_store(v[k], reinterpret_cast<v4f*>(obs_g + k * (kWave * 16)));
          obs_g += obs_stride;
        }
        if (mix_lds >= 0) {
          *reinterpret_cast<v4f*>(mix_g) = vm;
          mix_g += mix_stride;
        }
      }
      if (t == A.T) break;
      __syncthreads();  // X_t
      __syncthreads();  // Y_t
      const uint8_t* cur = buf[t & 1];
      if (obs_g) {
#pragma unroll
        for (int k = 0; k < SB::FULL; ++k) v[k] = *reinterpret_cast<const v4f*>(cur + (k * kWave + lane) * 16);
      }
      if (mix_lds >= 0) vm = *reinterpret_cast<const v4f*>(cur + mix_lds);
    }
  }
}

inline dim3 env_grid(uint32_t TE) { return dim3((TE + kWave - 1) / kWave); }

inline bool aligned16p(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The wave-specialised kernel needs whole waves and 16-byte aligned slices of every output.
template <int N>
inline bool ws_eligible(const RolloutArgs& A) {
  if (N > 3 || A.TE % kWave != 0) return false;
  if ((size_t(A.TE) * N) % 16 != 0) return false;  // action slices
  return aligned16p(A.obs_traj) && aligned16p(A.act_traj) && aligned16p(A.rew_traj) &&
         aligned16p(A.done_traj) && aligned16p(A.last_obs);
}

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
    if (A.ph.reward_mode == 1) {  // [T][TE][N] rewards: the general kernel
      hipLaunchKernelGGL((rollout_uniform_kernel<N, true>), env_grid(A.TE), dim3(kWave), 0, s, A);
      return;
    }
    if constexpr (N <= 3) {
      if (ws_eligible<N>(A)) {
        const uint32_t groups = A.TE / kWave;
        const uint32_t per_xcd = (groups + 7) / 8;
        hipLaunchKernelGGL(rollout_uniform_ws_kernel<N>, dim3(per_xcd * 8), dim3(2 * kWave), 0, s, A, groups, per_xcd);
        return;
      }
    }
    hipLaunchKernelGGL((rollout_uniform_kernel<N, false>), env_grid(A.TE), dim3(kWave), 0, s, A);
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
  // many agents: one lane per agent (the wide fused kernel without its policy) writes contiguous
  // pieces of the trajectory; the lane-per-env kernels below write one agent's rows at a time
  if (uniform_wide_supported(N) && launch_rollout_uniform_wide(N, A, s) == hipSuccess) return;
  MPE_DISPATCH_N(N, EnvLaunch<kN>::rollout(A, s));
}

}  // namespace mpe
