// Shared pieces of the fused-rollout kernels: tanh, wavefront-level LDS fence, Gumbel-max
// sampling.
#pragma once

#include "mpe_launch.h"

namespace mpe {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__host__ __device__ constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }

// tanh(x) = 1 - 2 / (exp(2x) + 1) on the hardware exp2 / rcp units.  Absolute error ~1e-7;
// saturates cleanly (exp2 -> inf gives 1, exp2 -> 0 gives -1).
__device__ __forceinline__ float fast_tanh(float x) {
  const float t = hw_exp2(x * (2.0f * kLog2e));
  return fmaf(-2.0f, hw_rcp(t + 1.0f), 1.0f);
}

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Barrier among the wavefronts of one sync group inside a larger block (several independent groups share a
// block's staged weights and must not wait for each other, so the block barrier is not the one to use).
// `arrived` is a counter in LDS, zeroed before the first use, that counts arrivals since the start of the
// kernel; `target` = (wavefronts per group) * (barriers so far), below 2^31 (the host bounds T).  Every
// wavefront of a block runs the same number of steps and none leaves early, and a block is resident as a
// whole, so each wait ends after at most one step of the slowest wavefront (microseconds).  The wait is
// bounded all the same: after `limit` polls (kBarrierSpinLimit unless the host lowers it to test this very
// path; each poll is a sleep of 64 clocks plus an LDS read: about a second in all) the wavefront gives up, sets the top bit of the counter, which lets every later wait of
// the group fall through at once, and raises *fault, a word the host reads before its next call on the
// handle.  A kernel therefore always runs to its end; after a give-up its results are invalid.
constexpr uint32_t kBarrierSpinLimit = 1u << 24;
constexpr uint32_t kBarrierBroken = 0x80000000u;

__device__ __forceinline__ void group_barrier(uint32_t* arrived, uint32_t target, int lane, uint32_t* fault,
                                              uint32_t limit) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  if (lane == 0) __hip_atomic_fetch_add(arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  uint32_t polls = 0;
  while (__hip_atomic_load(arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target) {
    __builtin_amdgcn_s_sleep(1);
    if (++polls >= limit) {
      if (lane == 0) {
        __hip_atomic_fetch_or(arrived, kBarrierBroken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (fault) __hip_atomic_store(fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
      break;
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Lane-per-agent pieces of the simple-spread step, shared by the kernels that keep one agent per lane with all
// positions of its env in registers.
// Transition of agent i under `act`: control force, contacts with the N - 1 other agents on the pre-step
// positions (the k-th OTHER agent is agent k for k < i, else k + 1: N - 1 evaluations on selected operands, in
// ascending agent order; a loop over all agents that skips a == i would run N masked evaluations), position
// with the old velocity, damped velocity.
template <int N>
__device__ __forceinline__ void agent_move(uint32_t act, int i, const Phys& ph, float& px, float& py, float& vx,
                                           float& vy, const float (&qx)[N], const float (&qy)[N]) {
  float fx = ph.accel * action_dir_x(act);
  float fy = ph.accel * action_dir_y(act);
#pragma unroll
  for (int k = 0; k < N - 1; ++k) {
    const bool up = k >= i;
    const float dx = px - (up ? qx[k + 1] : qx[k]);
    const float dy = py - (up ? qy[k + 1] : qy[k]);
    const float kf = contact_factor(dx, dy, ph);
    fx = fmaf(kf, dx, fx);
    fy = fmaf(kf, dy, fy);
  }
  px = fmaf(vx, ph.dt, px);
  py = fmaf(vy, ph.dt, py);
  vx = fmaf(fx, ph.dt_over_mass, vx * ph.keep);
  vy = fmaf(fy, ph.dt_over_mass, vy * ph.keep);
}

// Shared coverage reward of an env: minus the sum over landmarks of the distance to the nearest agent.
template <int N, int LA>
__device__ __forceinline__ float coverage_reward(const float (&qx)[N], const float (&qy)[N], const float (&lx)[LA],
                                                 const float (&ly)[LA]) {
  static_assert(LA >= N, "one landmark per agent");
  float r = 0.0f;
#pragma unroll
  for (int l = 0; l < N; ++l) {
    float best2 = INFINITY;
#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float dx = qx[a] - lx[l], dy = qy[a] - ly[l];
      best2 = fminf(best2, fmaf(dx, dx, dy * dy));
    }
    r -= hw_sqrt(best2);
  }
  return r;
}

// Other agents whose centre is strictly closer than 2 r to agent i (mixed per-agent reward).
template <int N>
__device__ __forceinline__ uint32_t overlap_count(int i, float px, float py, const float (&qx)[N], const float (&qy)[N],
                                                  const Phys& ph) {
  uint32_t overlaps = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a != i) {
      const float dx = px - qx[a], dy = py - qy[a];
      overlaps += fmaf(dx, dx, dy * dy) < ph.two_r_sq ? 1u : 0u;
    }
  }
  return overlaps;
}

// 4 x 4 transpose between register index and lane group (lane = 16 * group + j):
// out[c] at lane (j, g) = in[g] at lane (j, c).  No memory involved.
__device__ __forceinline__ void transpose_groups(uint32_t (&v)[4]) {
  const auto s0 = __builtin_amdgcn_permlane32_swap(v[0], v[2], false, false);   // upper half of v0 <-> lower half of v2
  const auto s1 = __builtin_amdgcn_permlane32_swap(v[1], v[3], false, false);
  const auto t0 = __builtin_amdgcn_permlane16_swap(s0[0], s1[0], false, false);  // odd 16-lane rows of v0 <-> even rows of v1
  const auto t1 = __builtin_amdgcn_permlane16_swap(s0[1], s1[1], false, false);
  v[0] = t0[0]; v[1] = t0[1]; v[2] = t1[0]; v[3] = t1[1];
}

// Gumbel-max over 5 logits: g = -ln(-ln u), u odd multiples of 2^-24 from two Philox blocks.
// ln = ln2 * log2 on the hardware unit (u >= 2^-24 is a normal number; -ln u is in
// [6e-8, 16.7], also normal), so v_k = z_k - ln2 * log2(-ln2 * log2(u_k)).
__device__ __forceinline__ uint32_t gumbel_argmax(const float (&z)[kNumActions], uint32_t seed,
                                                  uint32_t run, uint32_t env, uint32_t step, uint32_t agent) {
  const uint4 w0 = philox4x32_10(env, step, agent, kTagGumbel0, seed, run);
  const uint4 w1 = philox4x32_10(env, step, agent, kTagGumbel1, seed, run);
  const uint32_t w[kNumActions] = {w0.x, w0.y, w0.z, w0.w, w1.x};
  uint32_t best = 0;
  float best_v = -INFINITY;
#pragma unroll
  for (int k = 0; k < kNumActions; ++k) {
    const float u = word_to_open_uniform(w[k]);
    const float e = -kLn2 * hw_log2(u);               // -ln u  > 0
    const float v = fmaf(-kLn2, hw_log2(e), z[k]);     // z - ln(-ln u)
    if (v > best_v) { best_v = v; best = uint32_t(k); }
  }
  return best;
}

}  // namespace mpe
