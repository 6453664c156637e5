// Device-side building blocks of libmpe (gfx950 only): Philox4x32-10, the simple-spread
// transition of one environment held in registers, and the LDS-staged observation writer.
//
// The paper (JaxMARL, arXiv 2311.10090) states the MPE scenario in words only (Sec. 3.1
// "MPE", App. B.7) and its interface in App. C; the quantitative definition implemented
// here is the one documented in include/mpe.h and in the repository's design notes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpe {

typedef float v4f __attribute__((ext_vector_type(4)));  // native 16-byte vector (stays in VGPRs)
typedef float v2f __attribute__((ext_vector_type(2)));  // native 8-byte vector

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kNumActions = 5;

enum PhiloxTag : uint32_t { kTagResetPos = 0, kTagUniformAction = 1, kTagGumbel0 = 2, kTagGumbel1 = 3 };

// Physics constants, pre-combined on the host in double and rounded once to fp32.
struct Phys {
  float dt;
  float keep;           // 1 - damping
  float dt_over_mass;   // dt / mass
  float accel;
  float two_r;          // 2 * agent_radius
  float inv_margin;     // 1 / contact_margin
  float force_margin;   // contact_force * contact_margin
  int32_t max_ep;
  int32_t reward_mode;  // 0: one shared coverage reward per env; 1: one mixed reward per agent
  float local_ratio;    // mode 1: r_i = (1 - local_ratio) * coverage - local_ratio * overlaps_i
  float two_r_sq;       // (2 * agent_radius)^2
};

// Mixed per-agent reward from the shared coverage term and the number of other agents that
// overlap the agent (centre distance below 2 * agent_radius) after the step.
__device__ __forceinline__ float mixed_reward(float coverage, uint32_t overlaps, const Phys& ph) {
  return fmaf(-ph.local_ratio, float(overlaps), (1.0f - ph.local_ratio) * coverage);
}

// --------------------------------------------------------------------------------------
// Philox4x32 with 10 rounds (Salmon et al., SC'11).  key = (seed, run),
// counter = (env in run, absolute step, entity/agent, tag).
// --------------------------------------------------------------------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = uint64_t(0xD2511F53u) * c0;
    const uint64_t p1 = uint64_t(0xCD9E8D57u) * c2;
    const uint32_t n0 = uint32_t(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = uint32_t(p0 >> 32) ^ c3 ^ k1;
    c1 = uint32_t(p1);
    c3 = uint32_t(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

// 24-bit grid on [-1, 1): exact in fp32.
__device__ __forceinline__ float word_to_position(uint32_t w) {
  return float(w >> 8) * (1.0f / 8388608.0f) - 1.0f;
}
// Odd multiples of 2^-24 in (0, 1): exact in fp32, never 0 or 1.
__device__ __forceinline__ float word_to_open_uniform(uint32_t w) {
  return float(2u * (w >> 9) + 1u) * (1.0f / 16777216.0f);
}
__device__ __forceinline__ uint32_t word_to_action(uint32_t w) { return __umulhi(w, 5u); }

// --------------------------------------------------------------------------------------
// One environment in registers.
// --------------------------------------------------------------------------------------
template <int N>
struct Env {
  float px[N], py[N], vx[N], vy[N];  // agents
  float lx[N], ly[N];                // landmarks (L = N)
  int32_t ep;                        // steps since the last reset
};

template <int N>
__device__ __forceinline__ void reset_env(Env<N>& s, uint32_t seed, uint32_t run, uint32_t env,
                                          uint32_t step) {
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const uint4 w = philox4x32_10(env, step, uint32_t(e), kTagResetPos, seed, run);
    s.px[e] = word_to_position(w.x);
    s.py[e] = word_to_position(w.y);
    s.vx[e] = 0.0f;
    s.vy[e] = 0.0f;
  }
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const uint4 w = philox4x32_10(env, step, uint32_t(N + e), kTagResetPos, seed, run);
    s.lx[e] = word_to_position(w.x);
    s.ly[e] = word_to_position(w.y);
  }
  s.ep = 0;
}

// Hardware transcendentals (v_exp_f32 = 2^x, v_log_f32 = log2, v_rsq_f32, v_sqrt_f32, v_rcp_f32:
// about 1 ulp each, no denormal or range fix-ups).  Every use below stays inside their normal
// range, and the oracle comparison (1e-5 per transition) leaves two orders of magnitude of room.
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float hw_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float hw_rsq(float x) { return __builtin_amdgcn_rsqf(x); }
__device__ __forceinline__ float hw_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
__device__ __forceinline__ float hw_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// log(1 + exp(x)) as max(x, 0) + log(1 + exp(-|x|)); the second term is in (0, ln 2].
__device__ __forceinline__ float softplus(float x) {
  const float e = hw_exp2(-fabsf(x) * kLog2e);
  return fmaf(hw_log2(1.0f + e), kLn2, fmaxf(x, 0.0f));
}

// Contact force factor k of one agent pair with separation (dx, dy): the force on the first
// agent is k * (dx, dy), on the second -k * (dx, dy).
//   d = |delta| (clamped below at 1e-12, so coincident agents get zero force, no NaN)
//   k = contact_force * margin * softplus((2r - d) / margin) / d
__device__ __forceinline__ float contact_factor(float dx, float dy, const Phys& ph) {
  const float d2 = fmaxf(fmaf(dx, dx, dy * dy), 1e-24f);
  const float inv_d = hw_rsq(d2);
  const float d = d2 * inv_d;
  const float sp = softplus((ph.two_r - d) * ph.inv_margin);
  return ph.force_margin * sp * inv_d;
}

// Control force component from a discrete action (0 none, 1 -x, 2 +x, 3 -y, 4 +y), branch-free:
// two-bit fields of a constant hold direction + 1 for each action.
__device__ __forceinline__ float action_dir_x(uint32_t a) { return float((0x161u >> (2u * a)) & 3u) - 1.0f; }
__device__ __forceinline__ float action_dir_y(uint32_t a) { return float((0x215u >> (2u * a)) & 3u) - 1.0f; }

// One transition under actions a[0..N): control force, pairwise softplus contacts on the
// pre-step positions, position update with the old velocity, damped velocity update, shared
// coverage reward on the new positions (PER_AGENT: the N mixed rewards instead), episode
// counter, auto-reset keyed by step + 1.
template <int N, bool PER_AGENT = false>
__device__ __forceinline__ void transition(Env<N>& s, const uint32_t (&a)[N], const Phys& ph,
                                           uint32_t seed, uint32_t run, uint32_t env, uint32_t step,
                                           float (&reward)[PER_AGENT ? N : 1], bool& done) {
  float fx[N], fy[N];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    fx[i] = ph.accel * action_dir_x(a[i]);
    fy[i] = ph.accel * action_dir_y(a[i]);
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
#pragma unroll
    for (int j = i + 1; j < N; ++j) {
      const float dx = s.px[i] - s.px[j];
      const float dy = s.py[i] - s.py[j];
      const float k = contact_factor(dx, dy, ph);
      fx[i] = fmaf(k, dx, fx[i]);
      fy[i] = fmaf(k, dy, fy[i]);
      fx[j] = fmaf(-k, dx, fx[j]);
      fy[j] = fmaf(-k, dy, fy[j]);
    }
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    s.px[i] = fmaf(s.vx[i], ph.dt, s.px[i]);
    s.py[i] = fmaf(s.vy[i], ph.dt, s.py[i]);
    s.vx[i] = fmaf(fx[i], ph.dt_over_mass, s.vx[i] * ph.keep);
    s.vy[i] = fmaf(fy[i], ph.dt_over_mass, s.vy[i] * ph.keep);
  }
  float r = 0.0f;
#pragma unroll
  for (int l = 0; l < N; ++l) {
    float best2 = INFINITY;  // sqrt is monotone: take the min of squared distances, one sqrt
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const float dx = s.px[i] - s.lx[l];
      const float dy = s.py[i] - s.ly[l];
      best2 = fminf(best2, fmaf(dx, dx, dy * dy));
    }
    r -= hw_sqrt(best2);
  }
  if constexpr (PER_AGENT) {
    uint32_t ov[N];
#pragma unroll
    for (int i = 0; i < N; ++i) ov[i] = 0u;
#pragma unroll
    for (int i = 0; i < N; ++i) {
#pragma unroll
      for (int j = i + 1; j < N; ++j) {
        const float dx = s.px[i] - s.px[j];
        const float dy = s.py[i] - s.py[j];
        const uint32_t hit = fmaf(dx, dx, dy * dy) < ph.two_r_sq ? 1u : 0u;
        ov[i] += hit;
        ov[j] += hit;
      }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) reward[i] = mixed_reward(r, ov[i], ph);
  } else {
    reward[0] = r;
  }
  s.ep += 1;
  done = s.ep >= ph.max_ep;
  if (done) reset_env<N>(s, seed, run, env, step + 1u);
}

// --------------------------------------------------------------------------------------
// SoA state in HBM: pos_a, vel_a [2][N][TE]; pos_l [2][N][TE]; ep_step [TE].
// --------------------------------------------------------------------------------------
struct StatePtrs {
  float* pos_a;
  float* vel_a;
  float* pos_l;
  int32_t* ep_step;
};

template <int N>
__device__ __forceinline__ void load_state(Env<N>& s, const StatePtrs& st, size_t TE, size_t g) {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    s.px[i] = st.pos_a[(0 * N + i) * TE + g];
    s.py[i] = st.pos_a[(1 * N + i) * TE + g];
    s.vx[i] = st.vel_a[(0 * N + i) * TE + g];
    s.vy[i] = st.vel_a[(1 * N + i) * TE + g];
    s.lx[i] = st.pos_l[(0 * N + i) * TE + g];
    s.ly[i] = st.pos_l[(1 * N + i) * TE + g];
  }
  s.ep = st.ep_step[g];
}

template <int N>
__device__ __forceinline__ void store_state(const Env<N>& s, const StatePtrs& st, size_t TE, size_t g) {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    st.pos_a[(0 * N + i) * TE + g] = s.px[i];
    st.pos_a[(1 * N + i) * TE + g] = s.py[i];
    st.vel_a[(0 * N + i) * TE + g] = s.vx[i];
    st.vel_a[(1 * N + i) * TE + g] = s.vy[i];
    st.pos_l[(0 * N + i) * TE + g] = s.lx[i];
    st.pos_l[(1 * N + i) * TE + g] = s.ly[i];
  }
  st.ep_step[g] = s.ep;
}

template <int N>
__device__ __forceinline__ void zero_env(Env<N>& s) {
#pragma unroll
  for (int i = 0; i < N; ++i) {
    s.px[i] = s.py[i] = s.vx[i] = s.vy[i] = s.lx[i] = s.ly[i] = 0.0f;
  }
  s.ep = 0;
}

// --------------------------------------------------------------------------------------
// Observation writer.  A lane owns one env; its N*D floats are contiguous in the output
// ([g][agent][D]) but lanes are N*D*4 bytes apart, so direct stores would be dword
// scatters.  Instead each lane drops its float2 pairs into a per-wave LDS tile and the wave
// then streams the tile out with 16-byte (or 8-byte, when alignment forbids) stores that
// cover whole cache lines.
//   N <= 3 : the tile holds all agents, [lane][N*D]; the wave's output block is one
//            contiguous run of nvalid*N*D floats.
//   N  > 3 : one agent at a time, tile [lane][D]; rows of D floats, N*D apart in the output.
// The block is one wavefront, so __syncthreads() is only a wave-level LDS fence.
// --------------------------------------------------------------------------------------
template <int N>
struct ObsTile {
  static constexpr int D = 6 * N;
  static constexpr bool kFull = (N <= 3);
  static constexpr int kRow = kFull ? N * D : D;  // floats per lane in the tile
  static constexpr int kFloats = kWave * kRow;
};

// Agent i's observation of env state s, as D/2 float2 pairs written to row[0..D).
template <int N>
__device__ __forceinline__ void build_agent_obs(const Env<N>& s, int i, float2* row) {
  int c = 0;
  row[c++] = make_float2(s.vx[i], s.vy[i]);
  row[c++] = make_float2(s.px[i], s.py[i]);
#pragma unroll
  for (int l = 0; l < N; ++l) row[c++] = make_float2(s.lx[l] - s.px[i], s.ly[l] - s.py[i]);
#pragma unroll
  for (int j = 0; j < N; ++j) {
    if (j == i) continue;
    row[c++] = make_float2(s.px[j] - s.px[i], s.py[j] - s.py[i]);
  }
#pragma unroll
  for (int z = 0; z < N - 1; ++z) row[c++] = make_float2(0.0f, 0.0f);
}

// Stream `nfloats` (even) contiguous floats from the LDS tile to dst.  vec4 requires dst to
// be 16-byte aligned; otherwise 8-byte stores are used.  Generic (ragged) version.
// The stores are nontemporal: a wavefront's store covers whole cache lines that nothing reads
// again, and streaming them past the L2 leaves room there for the partial lines of the small
// outputs (actions, rewards, done flags) until their neighbours complete them (measured: 8-15 %
// on the HBM-bound rollouts; per-lane row stores at a stride are NOT made nontemporal, that
// is several times slower).
__device__ __forceinline__ void stream_out(const float* tile, float* dst, int nfloats, bool vec4, int lane) {
  if (vec4) {
    const int n4 = nfloats >> 2;
    for (int j = lane; j < n4; j += kWave)
      __builtin_nontemporal_store(reinterpret_cast<const v4f*>(tile)[j], reinterpret_cast<v4f*>(dst) + j);
    if ((nfloats & 2) && lane == 0)
      __builtin_nontemporal_store(reinterpret_cast<const v2f*>(tile)[nfloats / 2 - 1], reinterpret_cast<v2f*>(dst) + (nfloats / 2 - 1));
  } else {
    const int n2 = nfloats >> 1;
    for (int j = lane; j < n2; j += kWave)
      __builtin_nontemporal_store(reinterpret_cast<const v2f*>(tile)[j], reinterpret_cast<v2f*>(dst) + j);
  }
}

// Full-wave, 16-byte-aligned fast path: NF4 float4 per wave, known at compile time.  All LDS
// reads are issued before the first store so their latency overlaps instead of adding up.
template <int NF4>
__device__ __forceinline__ void stream_out_full(const float* tile, float* dst, int lane) {
  constexpr int kFullIters = NF4 / kWave;
  constexpr int kTail = NF4 % kWave;
  const v4f* src4 = reinterpret_cast<const v4f*>(tile) + lane;
  v4f* dst4 = reinterpret_cast<v4f*>(dst) + lane;
  v4f v[kFullIters > 0 ? kFullIters : 1];
  v4f vt = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int k = 0; k < kFullIters; ++k) v[k] = src4[k * kWave];
  if (kTail > 0 && lane < kTail) vt = src4[kFullIters * kWave];
#pragma unroll
  for (int k = 0; k < kFullIters; ++k) __builtin_nontemporal_store(v[k], &dst4[k * kWave]);
  if (kTail > 0 && lane < kTail) __builtin_nontemporal_store(vt, &dst4[kFullIters * kWave]);
}

// Write the observations of the wave's nvalid envs to dst_wave, which points at the row of the
// wave's first env inside an [env][N][D] slice.
template <int N>
__device__ __forceinline__ void emit_obs(const Env<N>& s, float* tile, float* dst_wave, int nvalid, int lane) {
  using OT = ObsTile<N>;
  constexpr int D = OT::D;
  if constexpr (OT::kFull) {
    float2* row = reinterpret_cast<float2*>(tile + lane * OT::kRow);
#pragma unroll
    for (int i = 0; i < N; ++i) build_agent_obs<N>(s, i, row + i * (D / 2));
    __syncthreads();
    const bool vec4 = (reinterpret_cast<uintptr_t>(dst_wave) & 15u) == 0;
    if (vec4 && nvalid == kWave) stream_out_full<kWave * N * D / 4>(tile, dst_wave, lane);
    else stream_out(tile, dst_wave, nvalid * N * D, vec4, lane);
    __syncthreads();
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      build_agent_obs<N>(s, i, reinterpret_cast<float2*>(tile + lane * D));
      __syncthreads();
      float* dst = dst_wave + i * D;
      const bool vec4 = (D % 4 == 0) && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
      if (vec4) {
        constexpr int Q = (D % 4 == 0) ? D / 4 : 1;
        if (nvalid == kWave) {
          v4f v[Q];
#pragma unroll
          for (int k = 0; k < Q; ++k) v[k] = reinterpret_cast<const v4f*>(tile)[k * kWave + lane];
#pragma unroll
          for (int k = 0; k < Q; ++k) {
            const int j = k * kWave + lane, e = j / Q, q = j - e * Q;
            reinterpret_cast<v4f*>(dst + size_t(e) * N * D)[q] = v[k];
          }
        } else {
          for (int j = lane; j < nvalid * Q; j += kWave) {
            const int e = j / Q, q = j - e * Q;
            reinterpret_cast<float4*>(dst + size_t(e) * N * D)[q] = reinterpret_cast<const float4*>(tile + e * D)[q];
          }
        }
      } else {
        constexpr int Q = D / 2;
        for (int j = lane; j < nvalid * Q; j += kWave) {
          const int e = j / Q, q = j - e * Q;
          reinterpret_cast<float2*>(dst + size_t(e) * N * D)[q] = reinterpret_cast<const float2*>(tile + e * D)[q];
        }
      }
      __syncthreads();
    }
  }
}

}  // namespace mpe
