// Device helpers of the predator-prey ("simple tag") scenario of the MPE family (paper App. B.7, Sec. 3.1
// "MPE"): the shape of an instance, the contact law, the boundary penalty, the reset draw and the
// observation row.  Shared by the scenario's own kernels and by the recurrent-policy kernel.
#pragma once

#include "mpe_policy_common.h"

namespace mpe {

namespace {

template <int N_, int L_, int G_>
struct TagShape {
  static constexpr int N = N_, L = L_, G = G_, A = N_ - G_;   // A adversaries first, then G good agents
  static constexpr int D = 4 + 2 * L_ + 2 * (N_ - 1) + 2 * G_;
  static constexpr bool kWaveLocal = (64 % N_) == 0;          // the rows of an env lie in one wavefront
  static_assert(G_ >= 1 && A >= 1 && L_ >= 0 && D % 2 == 0, "roles");
};

// Contact force factor k of a pair with separation (dx, dy) and contact distance dmin: the force
// on the first entity is k * (dx, dy).
__device__ __forceinline__ float tag_contact(float dx, float dy, float dmin, const TagPhys& tg) {
  const float d2 = fmaxf(fmaf(dx, dx, dy * dy), 1e-24f);
  const float inv_d = hw_rsq(d2);
  const float d = d2 * inv_d;
  return tg.force_margin * softplus((dmin - d) * tg.inv_margin) * inv_d;
}

// Boundary penalty of a good agent for one coordinate, u = |coordinate|.
__device__ __forceinline__ float tag_bound(float u) {
  const float lin = (u - 0.9f) * 10.0f;
  const float ex = fminf(hw_exp2((2.0f * u - 2.0f) * kLog2e), 10.0f);
  return u < 0.9f ? 0.0f : (u < 1.0f ? lin : ex);
}

// Fresh positions of every entity of an env for the episode that starts at `step`.
template <typename S>
__device__ __forceinline__ void tag_draw_positions(float (&qx)[S::N], float (&qy)[S::N], float (&lx)[S::L + 1],
                                                   float (&ly)[S::L + 1], uint32_t env, uint32_t step,
                                                   uint32_t seed, uint32_t run) {
#pragma unroll
  for (int a = 0; a < S::N; ++a) {
    const uint4 w = philox4x32_10(env, step, uint32_t(a), kTagResetPos, seed, run);
    qx[a] = word_to_position(w.x);
    qy[a] = word_to_position(w.y);
  }
#pragma unroll
  for (int k = 0; k < S::L; ++k) {
    const uint4 w = philox4x32_10(env, step, uint32_t(S::N + k), kTagResetPos, seed, run);
    lx[k] = word_to_position(w.x) * 0.9f;   // obstacles start inside [-0.9, 0.9): one fp32 product
    ly[k] = word_to_position(w.y) * 0.9f;
  }
}

// Observation row of agent i: own velocity, own position, landmarks and other agents relative,
// velocities of the other good agents, zero padding (good agents see one velocity fewer).
template <typename S>
__device__ __forceinline__ void tag_write_row(float2* row, int i, float px, float py, float vx, float vy,
                                              const float (&qx)[S::N], const float (&qy)[S::N],
                                              const float (&lx)[S::L + 1], const float (&ly)[S::L + 1],
                                              const float (&gvx)[S::G], const float (&gvy)[S::G]) {
  int c = 0;
  row[c++] = make_float2(vx, vy);
  row[c++] = make_float2(px, py);
#pragma unroll
  for (int k = 0; k < S::L; ++k) row[c++] = make_float2(lx[k] - px, ly[k] - py);
#pragma unroll
  for (int a = 0; a < S::N; ++a) {
    if (a != i) row[c++] = make_float2(qx[a] - px, qy[a] - py);
  }
#pragma unroll
  for (int k = 0; k < S::G; ++k) {
    if (S::A + k != i) row[c++] = make_float2(gvx[k], gvy[k]);
  }
  if (i >= S::A) row[S::D / 2 - 1] = make_float2(0.0f, 0.0f);
}

// The constants of an agent's role (adversaries come first).
struct TagRole {
  int role;            // 0 adversary, 1 good agent
  float radius, gain, limit, limit_sq;
};
template <typename S>
__device__ __forceinline__ TagRole tag_role(int i, const TagPhys& tg) {
  TagRole r;
  r.role = i < S::A ? 0 : 1;
  r.radius = r.role == 0 ? tg.radius[0] : tg.radius[1];
  r.gain = r.role == 0 ? tg.gain[0] : tg.gain[1];
  r.limit = r.role == 0 ? tg.limit[0] : tg.limit[1];
  r.limit_sq = r.role == 0 ? tg.limit_sq[0] : tg.limit_sq[1];
  return r;
}

// Transition of agent i under action `act`: control force, contacts with the other agents and with the obstacle
// landmarks on the pre-step positions, position with the old velocity, damped velocity, speed limit.
template <typename S>
__device__ __forceinline__ void tag_move(uint32_t act, int i, const TagRole& me, const TagPhys& tg, float& px, float& py,
                                         float& vx, float& vy, const float (&qx)[S::N], const float (&qy)[S::N],
                                         const float (&lx)[S::L + 1], const float (&ly)[S::L + 1]) {
  constexpr int N = S::N, NA = S::A;
  float fx = me.gain * action_dir_x(act);
  float fy = me.gain * action_dir_y(act);
  // the k-th OTHER agent is agent k (k < i) or k + 1: N - 1 evaluations with selected operands, in
  // ascending agent order (a loop over all agents that skips a == i runs N masked evaluations)
#pragma unroll
  for (int k = 0; k < N - 1; ++k) {
    const bool up = k >= i;
    const float ox = up ? qx[k + 1] : qx[k], oy = up ? qy[k + 1] : qy[k];
    const float r_lo = tg.radius[k < NA ? 0 : 1], r_hi = tg.radius[k + 1 < NA ? 0 : 1];
    const float orad = ((k < NA) == (k + 1 < NA)) ? r_lo : (up ? r_hi : r_lo);
    const float dx = px - ox, dy = py - oy;
    const float kf = tag_contact(dx, dy, me.radius + orad, tg);
    fx = fmaf(kf, dx, fx);
    fy = fmaf(kf, dy, fy);
  }
#pragma unroll
  for (int l = 0; l < S::L; ++l) {
    const float dx = px - lx[l], dy = py - ly[l];
    const float k = tag_contact(dx, dy, me.radius + tg.lm_radius, tg);
    fx = fmaf(k, dx, fx);
    fy = fmaf(k, dy, fy);
  }
  px = fmaf(vx, tg.dt, px);
  py = fmaf(vy, tg.dt, py);
  vx = fmaf(fx, tg.dt_over_mass, vx * tg.keep);
  vy = fmaf(fy, tg.dt_over_mass, vy * tg.keep);
  const float s2 = fmaf(vx, vx, vy * vy);
  if (s2 > me.limit_sq) {
    const float k = me.limit * hw_rsq(s2);
    vx *= k;
    vy *= k;
  }
}

// Reward of agent i on the new positions q (its own: px, py): every adversary gets 10 per touching (good,
// adversary) pair, a good agent loses 10 per adversary touching it and pays the boundary penalty.
template <typename S>
__device__ __forceinline__ float tag_reward(int i, const TagRole& me, const TagPhys& tg, float px, float py,
                                            const float (&qx)[S::N], const float (&qy)[S::N]) {
  uint32_t caught = 0, hits = 0;
#pragma unroll
  for (int a = 0; a < S::A; ++a) {
#pragma unroll
    for (int b = S::A; b < S::N; ++b) {
      const float dx = qx[a] - qx[b], dy = qy[a] - qy[b];
      const uint32_t touch = fmaf(dx, dx, dy * dy) < tg.touch_sq ? 1u : 0u;
      caught += touch;
      hits += b == i ? touch : 0u;
    }
  }
  const float r_good = -10.0f * float(hits) - tag_bound(fabsf(px)) - tag_bound(fabsf(py));
  return me.role == 0 ? 10.0f * float(caught) : r_good;
}

// The same observation row into a register array (every index a compile-time constant): entries
// 0 .. D - 1 of o; the caller zeroes what lies beyond.
template <typename S, int W>
__device__ __forceinline__ void tag_obs_regs(float (&o)[W], int i, float px, float py, float vx, float vy,
                                             const float (&qx)[S::N], const float (&qy)[S::N],
                                             const float (&lx)[S::L + 1], const float (&ly)[S::L + 1],
                                             const float (&gvx)[S::G], const float (&gvy)[S::G]) {
  static_assert(W >= S::D, "row buffer");
  o[0] = vx; o[1] = vy; o[2] = px; o[3] = py;
#pragma unroll
  for (int k = 0; k < S::L; ++k) { o[4 + 2 * k] = lx[k] - px; o[5 + 2 * k] = ly[k] - py; }
  // the k-th OTHER agent is agent k (k < i) or k + 1
#pragma unroll
  for (int k = 0; k < S::N - 1; ++k) {
    const bool up = k >= i;
    o[4 + 2 * S::L + 2 * k] = (up ? qx[k + 1] : qx[k]) - px;
    o[5 + 2 * S::L + 2 * k] = (up ? qy[k + 1] : qy[k]) - py;
  }
  // velocities of the other good agents: an adversary sees all G, good agent gi = i - A sees the others
  // and a zero pair at the end
  constexpr int base = 4 + 2 * S::L + 2 * (S::N - 1);
  const int gi = i - S::A;
#pragma unroll
  for (int k = 0; k < S::G; ++k) {
    float ax, ay;
    if (k + 1 < S::G) {
      const bool up = gi >= 0 && k >= gi;
      ax = up ? gvx[k + 1] : gvx[k];
      ay = up ? gvy[k + 1] : gvy[k];
    } else {
      ax = gvx[k];
      ay = gvy[k];
    }
    const bool pad = gi >= 0 && k == S::G - 1;
    o[base + 2 * k] = pad ? 0.0f : ax;
    o[base + 2 * k + 1] = pad ? 0.0f : ay;
  }
}

}  // namespace

}  // namespace mpe
