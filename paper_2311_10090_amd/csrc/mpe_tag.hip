// Predator-prey ("simple tag") scenario of the MPE family (paper App. B.7: every scenario of the
// family is implemented; Sec. 3.1 "MPE"): reset, single step, and the persistent T-step rollout
// with uniform actions or with the fused policy, fp32 (three-term fp16 operand split) or bf16 (App. G: two tanh layers of width 64).
//
// Mapping: one lane per agent row, a block is 64 envs = N wavefronts (as in the fused simple-spread
// kernel).  A lane keeps its own agent's position and velocity, the positions of all agents of its
// env and the obstacle landmarks in registers; per step the agents of an env exchange their new
// position and velocity through LDS (one barrier: wavefront-local when 64 % N == 0, the block
// barrier otherwise).  Every lane writes its own observation row into an LDS tile; a wavefront's
// 64 rows are one contiguous piece of the trajectory and leave with 16-byte stores over whole
// cache lines.  Rewards are per agent, so every lane stores its own.
#include "mpe_mlp64.h"
#include "mpe_tag_device.h"

namespace mpe {

namespace {

// kPolicy / kPolicyBf: fp32 (split-operand) / bf16 policy.  kPolicyAc / kPolicyAcBf: the policy plus a critic
// of the same shape with one output: log-probability of the sampled action and value per agent and step.
enum TagMode : int { kGiven = 0, kUniform = 1, kPolicy = 2, kPolicyBf = 3, kPolicyAc = 4, kPolicyAcBf = 5 };
constexpr bool mode_is_ac(int mode) { return mode == kPolicyAc || mode == kPolicyAcBf; }
constexpr bool mode_is_bf(int mode) { return mode == kPolicyBf || mode == kPolicyAcBf; }

// EB = envs per block.  Plain rollouts: 64.  Actor-critic: both packed images (79 KB) are staged per block,
// so a block is 8 wavefronts where the shape allows it (wavefront-local shapes need no block barrier).
// ROWS = the block's agent rows, rounded up to whole wavefronts of RW rows (only 16-env blocks of 3 agents
// have such padding rows: 48 -> 64; no env owns them and nothing of them leaves the block).
template <typename S, int MODE, int EB = 64, int RW = 64>
struct TagSmem {
  static constexpr int ROWS = (EB * S::N + RW - 1) / RW * RW;
  static constexpr bool kAc = mode_is_ac(MODE);
  static constexpr bool kHasPolicy = MODE == kPolicy || MODE == kPolicyBf || kAc;
  using P = PkT<mode_is_bf(MODE), (S::D > 16)>;
  // plain policy: W1A, W2A, then the biases (W3A lives in registers); actor-critic: the whole image of
  // the policy, then the whole image of the critic (their W3A are re-read every step)
  static constexpr size_t OFF_BIAS = kAc ? P::OFF_BIAS : (kHasPolicy ? P::LDS_BYTES : 0);
  static constexpr size_t OFF_CRITIC = P::RUN_BYTES;                                    // kAc only
  static constexpr size_t OFF_OBS = kAc ? 2 * P::RUN_BYTES : OFF_BIAS + (kHasPolicy ? P::BIAS_BYTES : 0);
  static constexpr size_t OBS = size_t(ROWS) * S::D * 4 + 64;   // + zeroed tail: layer 1 reads 16 (32) cols
  static constexpr size_t OFF_XCH = OFF_OBS + OBS;              // [parity][ROWS] float4 (px, py, vx, vy)
  static constexpr size_t OFF_VALUE = OFF_XCH + size_t(S::kWaveLocal ? 1 : 2) * ROWS * 16;   // kAc: [ROWS] float
  static constexpr size_t TOTAL = OFF_VALUE + (kAc ? size_t(ROWS) * 4 : 0);
  static_assert(OFF_OBS % 16 == 0 && OFF_XCH % 16 == 0 && P::RUN_BYTES % 16 == 0, "alignment");
  static_assert(TOTAL <= 160 * 1024, "LDS budget");
};

template <typename S>
__global__ __launch_bounds__(64 * S::N) void tag_reset_kernel(StatePtrs st, uint32_t TE, uint32_t E, uint32_t seed,
                                                              float* __restrict__ obs) {
  constexpr int N = S::N, L = S::L, D = S::D;
  const int tid = threadIdx.x;
  const int el = tid / N, i = tid - el * N;
  const size_t g = size_t(blockIdx.x) * 64 + el;
  if (g >= TE) return;
  const uint32_t run = uint32_t(g) / E, env = uint32_t(g) - run * E;
  float qx[N], qy[N], lx[L + 1], ly[L + 1], gvx[S::G], gvy[S::G];
  tag_draw_positions<S>(qx, qy, lx, ly, env, 0u, seed, run);
#pragma unroll
  for (int k = 0; k < S::G; ++k) gvx[k] = gvy[k] = 0.0f;
  float px = 0.0f, py = 0.0f;
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a == i) { px = qx[a]; py = qy[a]; }
  }
  st.pos_a[(0 * N + i) * size_t(TE) + g] = px;
  st.pos_a[(1 * N + i) * size_t(TE) + g] = py;
  st.vel_a[(0 * N + i) * size_t(TE) + g] = 0.0f;
  st.vel_a[(1 * N + i) * size_t(TE) + g] = 0.0f;
  if (i == 0) {
#pragma unroll
    for (int k = 0; k < L; ++k) {
      st.pos_l[(0 * L + k) * size_t(TE) + g] = lx[k];
      st.pos_l[(1 * L + k) * size_t(TE) + g] = ly[k];
    }
    st.ep_step[g] = 0;
  }
  if (obs) {
    float2 row[D / 2];
#pragma unroll
    for (int c = 0; c < D / 2; ++c) row[c] = make_float2(0.0f, 0.0f);
    tag_write_row<S>(row, i, px, py, 0.0f, 0.0f, qx, qy, lx, ly, gvx, gvy);
    float2* dst = reinterpret_cast<float2*>(obs + (g * N + i) * D);
#pragma unroll
    for (int c = 0; c < D / 2; ++c) dst[c] = row[c];
  }
}

//
// RW = rows per wavefront: 64 (one lane per row), or 32 for small batches of the policy modes: twice the
// wavefronts, one pair of 16-row tiles each; lanes 32..63 are exact clones of lanes 0..31 (same row, same
// inputs, same arithmetic, so their LDS writes repeat the same values) that store nothing to global memory.
// Wavefronts per SIMD the register budget is set for: three blocks per CU for the plain policy kernels whose
// LDS allows it, one block otherwise.
template <typename S, int MODE, int EB, int RW>
struct TagOccupancy {
  static constexpr bool kThree =
      (MODE == kPolicy || MODE == kPolicyBf) && RW == 64 && 3 * TagSmem<S, MODE, EB, RW>::TOTAL <= 160 * 1024;
  static constexpr int kWavesPerSimd = kThree ? 3 : 1;
};

template <typename S, int MODE, int EB = 64, int RW = 64>
__global__ __launch_bounds__((EB * S::N + RW - 1) / RW * 64, (TagOccupancy<S, MODE, EB, RW>::kWavesPerSimd)) void tag_rollout_kernel(
    TagArgs TA, const uint8_t* __restrict__ packed, const uint8_t* __restrict__ packed_critic, int per_run_weights,
    uint32_t groups, uint32_t groups_per_xcd) {
  using M = TagSmem<S, MODE, EB, RW>;
  constexpr bool AC = mode_is_ac(MODE), BF = mode_is_bf(MODE);
  static_assert(EB <= 64 || S::kWaveLocal, "larger blocks only where wavefronts never exchange data");
  static_assert(RW == 64 || (RW == 32 && (!S::kWaveLocal || 32 % S::N == 0)), "rows per wavefront");
  using Net = NetShape<S::D, S::D <= 32 ? S::D : 32>;
  constexpr int N = S::N, L = S::L, G = S::G, NA = S::A, D = S::D, ROWS = M::ROWS, THREADS = ROWS * (64 / RW);
  constexpr bool kPadded = ROWS != EB * N;
  static_assert(THREADS % 64 == 0, "block must be whole wavefronts");
  const RolloutArgs& A = TA.r;
  const TagPhys& tg = TA.tg;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  float* tile = reinterpret_cast<float*>(smem + M::OFF_OBS);
  float4* xch = reinterpret_cast<float4*>(smem + M::OFF_XCH);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int tid = wave * RW + (lane & (RW - 1));     // this lane's row
  const int el_row = tid / N, i = tid - el_row * N;  // env within block, agent
  const bool in_block = !kPadded || el_row < EB;     // false for padding rows: they shadow env 0 of the block
  const int el = in_block ? el_row : 0;
  const size_t TE = A.TE;
  // block b runs on XCD b % 8: give each XCD one contiguous range of env groups
  const uint32_t grp = (blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3);
  if (grp >= groups) return;  // whole block, before any barrier
  const size_t g0 = size_t(grp) * EB;
  const size_t g = g0 + el;
  const bool in_range = in_block && g < TE;
  const bool valid = in_range && lane < RW;          // the lane that stores this row's outputs
  const uint32_t gc = in_range ? uint32_t(g) : uint32_t(g0);
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;
  const size_t left = TE - g0;
  const int nvalid = left < size_t(EB) ? int(left) : EB;
  const int wave_rows = min(max(nvalid * N - wave * RW, 0), RW);   // rows of this wavefront that exist

  // ---- policy: W1A, W2A and the biases in LDS, W3A in registers (the run of the block's first env);
  // actor-critic: both whole images in LDS, W3A of the network in use re-read from there
  using Pk = typename M::P;
  [[maybe_unused]] auto load_w3 = [&](const uint8_t* image) {
    W3Terms w;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if constexpr (BF || Net::kRowTerms) {
        w.s[s].h = reinterpret_cast<const bf16x8*>(image + Pk::OFF_W3A)[s * 64 + lane];
      } else {
        const bf16x8* src = reinterpret_cast<const bf16x8*>(image + Pk::OFF_W3A) + s * 3 * 64 + lane;
        w.s[s].h = src[0];
        w.s[s].m = src[64];
        w.s[s].l = src[128];
      }
    }
    return w;
  };
  W3Terms w3;
  if constexpr (M::kHasPolicy) {
    const size_t run_off = per_run_weights ? size_t(uint32_t(g0) / A.E) * Pk::RUN_BYTES : 0;
    const uint8_t* run_weights = packed + run_off;
    const uint4* src = reinterpret_cast<const uint4*>(run_weights);
    uint4* dst = reinterpret_cast<uint4*>(smem);
    if constexpr (AC) {
      for (int k = threadIdx.x; k < int(Pk::RUN_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* csrc = reinterpret_cast<const uint4*>(packed_critic + run_off);
      uint4* cdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC);
      for (int k = threadIdx.x; k < int(Pk::RUN_BYTES / 16); k += THREADS) cdst[k] = csrc[k];
    } else {
      w3 = load_w3(run_weights);
      for (int k = threadIdx.x; k < int(Pk::LDS_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + Pk::OFF_BIAS);
      uint4* bdst = reinterpret_cast<uint4*>(smem + M::OFF_BIAS);
      for (int k = threadIdx.x; k < int(Pk::BIAS_BYTES / 16); k += THREADS) bdst[k] = bsrc[k];
    }
  }
  if (threadIdx.x < 16) tile[ROWS * D + threadIdx.x] = 0.0f;

  // ---- registers: own agent, all agents' positions, good agents' velocities, landmarks
  const TagRole me = tag_role<S>(i, tg);
  float px = 0.0f, py = 0.0f, vx = 0.0f, vy = 0.0f;
  float qx[N], qy[N], lx[L + 1], ly[L + 1], gvx[G], gvy[G];
  int32_t ep = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) qx[a] = qy[a] = 0.0f;
#pragma unroll
  for (int k = 0; k < L + 1; ++k) lx[k] = ly[k] = 0.0f;
#pragma unroll
  for (int k = 0; k < G; ++k) gvx[k] = gvy[k] = 0.0f;
  if (in_range) {
#pragma unroll
    for (int a = 0; a < N; ++a) {
      qx[a] = A.st.pos_a[(0 * N + a) * TE + g];
      qy[a] = A.st.pos_a[(1 * N + a) * TE + g];
    }
#pragma unroll
    for (int k = 0; k < L; ++k) {
      lx[k] = A.st.pos_l[(0 * L + k) * TE + g];
      ly[k] = A.st.pos_l[(1 * L + k) * TE + g];
    }
#pragma unroll
    for (int k = 0; k < G; ++k) {
      gvx[k] = A.st.vel_a[(0 * N + NA + k) * TE + g];
      gvy[k] = A.st.vel_a[(1 * N + NA + k) * TE + g];
    }
    vx = A.st.vel_a[(0 * N + i) * TE + g];
    vy = A.st.vel_a[(1 * N + i) * TE + g];
    ep = A.st.ep_step[g];
  }
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a == i) { px = qx[a]; py = qy[a]; }
  }
  float2* my_row = reinterpret_cast<float2*>(tile + tid * D);
  tag_write_row<S>(my_row, i, px, py, vx, vy, qx, qy, lx, ly, gvx, gvy);
  __syncthreads();  // weights, biases, zero tail staged

  const size_t wave_row0 = (g0 * N + size_t(wave) * RW) * D;   // float offset of this wavefront's rows in a slice
  float* obs_p = A.obs_traj ? A.obs_traj + wave_row0 : nullptr;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  const size_t row_off = size_t(gc) * N + i;          // index of this agent inside a time slice
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  uint32_t step = A.abs_step;
  const float* wtile = tile + wave * (RW * D);        // this wavefront's rows

  [[maybe_unused]] float* values = reinterpret_cast<float*>(smem + M::OFF_VALUE);   // AC: critic value per row
  [[maybe_unused]] float* logp_base = A.logp_traj;
  [[maybe_unused]] float* value_base = A.value_traj;
  // Critic forward of this wavefront's rows into values[] (its rows only: no other wavefront reads them).
  [[maybe_unused]] auto critic_rows = [&]() {
    if constexpr (AC) {
      const uint8_t* csm = smem + M::OFF_CRITIC;
      const float* cbias = reinterpret_cast<const float*>(csm + Pk::OFF_BIAS);
#pragma unroll 1
      for (int pr = 0; pr < RW / 32; ++pr) {
        float* rows = tile + (wave * RW + pr * 32) * D;
        float* vals = values + wave * RW + pr * 32;
        const W3Terms wc = load_w3(csm);
        if constexpr (BF) policy_pair_bf<Net, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
        else policy_pair<Net, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
      }
    }
  };

  auto flush_rows = [&](float* dst) {
    const bool vec4 = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
    if (vec4 && wave_rows == RW) stream_out_full<RW * D / 4>(wtile, dst, lane);
    else stream_out(wtile, dst, wave_rows * D, vec4, lane);
  };

  for (int t = 0; t < A.T; ++t, ++step) {
    wave_sync();  // this wavefront's rows of the tile are complete
    if (obs_p) {
      flush_rows(obs_p);
      obs_p += TE * (N * D);
    }
    // ---- action
    uint32_t act;
    if constexpr (MODE == kGiven) {
      const uint32_t v = in_range ? TA.actions_in[row_off] : 0u;
      act = v < uint32_t(kNumActions) ? v : 0u;
    } else if constexpr (MODE == kUniform) {
      act = word_to_action(philox4x32_10(env, step, uint32_t(i), kTagUniformAction, A.seed, run).x);
    } else {
      const float* bias = reinterpret_cast<const float*>(smem + M::OFF_BIAS);
      // the critic first (it leaves the rows untouched), then the policy, whose logits replace the
      // first columns of the rows
      if constexpr (AC) critic_rows();
#pragma unroll 1
      for (int pr = 0; pr < RW / 32; ++pr) {
        float* rows = tile + (wave * RW + pr * 32) * D;
        if constexpr (AC) w3 = load_w3(smem);
        if constexpr (BF) policy_pair_bf<Net>(smem, bias, w3, rows, rows + 16 * D, lane);
        else policy_pair<Net>(smem, bias, w3, rows, rows + 16 * D, lane);
      }
      wave_sync();
      float z[kNumActions];
#pragma unroll
      for (int k = 0; k < kNumActions; ++k) z[k] = tile[tid * D + k];
      if constexpr (!BF && Net::kRowTerms) z[4] = (z[4] + tile[tid * D + 5]) + tile[tid * D + 6];
      act = gumbel_argmax(z, A.seed, run, env, step, uint32_t(i));
      if constexpr (AC) {
        // log pi(act | obs) = z_act - max - ln sum exp(z - max)
        float zmax = z[0], zact = z[0];
#pragma unroll
        for (int k = 1; k < kNumActions; ++k) {
          zmax = fmaxf(zmax, z[k]);
          zact = act == uint32_t(k) ? z[k] : zact;
        }
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < kNumActions; ++k) sum += hw_exp2((z[k] - zmax) * kLog2e);
        if (logp_base) {
          if (valid) logp_base[row_off] = (zact - zmax) - kLn2 * hw_log2(sum);
          logp_base += TE * N;
        }
        if (value_base) {
          if (valid) value_base[row_off] = values[tid];
          value_base += TE * N;
        }
      }
    }
    if (act_base) {
      if (valid) act_base[row_off] = uint8_t(act);
      act_base += TE * N;
    }

    // ---- transition of this lane's agent
    tag_move<S>(act, i, me, tg, px, py, vx, vy, qx, qy, lx, ly);
    float4* slot = xch + (S::kWaveLocal ? 0 : (t & 1) * ROWS);
    slot[tid] = make_float4(px, py, vx, vy);
    // new positions and velocities of every agent of this env are visible
    if constexpr (S::kWaveLocal) wave_sync(); else __syncthreads();
#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float4 p = slot[el * N + a];
      qx[a] = p.x;
      qy[a] = p.y;
      if (a >= NA) {
        gvx[a - NA] = p.z;
        gvy[a - NA] = p.w;
      }
    }
    if constexpr (S::kWaveLocal) wave_sync();   // the slots are rewritten in the next step

    // ---- rewards on the new positions
    if (rew_base) {
      const float r = tag_reward<S>(i, me, tg, px, py, qx, qy);
      if (valid) rew_base[row_off] = r;
      rew_base += TE * N;
    }
    ep += 1;
    const bool done = ep >= tg.max_ep;
    if (done_base) {
      if (env_writer) done_base[gc] = done ? 1 : 0;
      done_base += TE;
    }
    if (done) {
      // new episode keyed by step + 1; every lane regenerates the whole env (1 step in max_ep).
      // The empty asm keeps the env-dependent first Philox round out of the step loop's preamble.
      uint32_t env_r = env;
      asm volatile("" : "+v"(env_r));
      tag_draw_positions<S>(qx, qy, lx, ly, env_r, step + 1u, A.seed, run);
#pragma unroll
      for (int a = 0; a < N; ++a) {
        if (a == i) { px = qx[a]; py = qy[a]; }
      }
#pragma unroll
      for (int k = 0; k < G; ++k) gvx[k] = gvy[k] = 0.0f;
      vx = vy = 0.0f;
      ep = 0;
    }
    tag_write_row<S>(my_row, i, px, py, vx, vy, qx, qy, lx, ly, gvx, gvy);
  }
  if (A.last_obs) {
    wave_sync();
    flush_rows(A.last_obs + wave_row0);
  }
  if constexpr (AC) {
    if (A.last_value) {   // value of the observation after the last step
      wave_sync();
      critic_rows();
      wave_sync();
      if (valid) A.last_value[row_off] = values[tid];
    }
  }

  // ---- state back to HBM
  if (valid) {
    A.st.pos_a[(0 * N + i) * TE + g] = px;
    A.st.pos_a[(1 * N + i) * TE + g] = py;
    A.st.vel_a[(0 * N + i) * TE + g] = vx;
    A.st.vel_a[(1 * N + i) * TE + g] = vy;
    if (i == 0) {
#pragma unroll
      for (int k = 0; k < L; ++k) {
        A.st.pos_l[(0 * L + k) * TE + g] = lx[k];
        A.st.pos_l[(1 * L + k) * TE + g] = ly[k];
      }
      A.st.ep_step[g] = ep;
    }
  }
}

template <typename S, int MODE, int EB = 64, int RW = 64>
hipError_t tag_rollout_impl(const TagArgs& A, const void* packed, const void* packed_critic, hipStream_t s) {
  using M = TagSmem<S, MODE, EB, RW>;
  auto kern = tag_rollout_kernel<S, MODE, EB, RW>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (hipError_t e = allow_lds(reinterpret_cast<const void*>(kern), M::TOTAL, lds_allowed); e != hipSuccess) return e;
  const uint32_t groups = (A.r.TE + EB - 1) / EB;
  const uint32_t per_xcd = (groups + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(M::ROWS * (64 / RW)), M::TOTAL, s, A,
                     static_cast<const uint8_t*>(packed), static_cast<const uint8_t*>(packed_critic),
                     int(A.r.TE != A.r.E), groups, per_xcd);
  return hipGetLastError();
}

// One policy mode at one block shape: the critic's image goes along in the actor-critic modes only.
template <typename S, int EB, int RW, bool AC>
hipError_t tag_policy_impl(int mode, const TagArgs& A, const void* packed, const void* packed_critic, hipStream_t s) {
  if constexpr (AC) {
    if (mode == kPolicyAc) return tag_rollout_impl<S, kPolicyAc, EB, RW>(A, packed, packed_critic, s);
    if (mode == kPolicyAcBf) return tag_rollout_impl<S, kPolicyAcBf, EB, RW>(A, packed, packed_critic, s);
  } else {
    if (mode == kPolicy) return tag_rollout_impl<S, kPolicy, EB, RW>(A, packed, nullptr, s);
    if (mode == kPolicyBf) return tag_rollout_impl<S, kPolicyBf, EB, RW>(A, packed, nullptr, s);
  }
  return hipErrorInvalidValue;
}

template <typename S>
hipError_t tag_launch(int mode, const TagArgs& A, const void* packed, const void* packed_critic, hipStream_t s,
                      const char** why) {
  if (mode == kGiven) return tag_rollout_impl<S, kGiven>(A, nullptr, nullptr, s);
  if (mode == kUniform) return tag_rollout_impl<S, kUniform>(A, nullptr, nullptr, s);
  if constexpr (S::D <= 32) {
    // actor-critic: both images are staged per block; 8 wavefronts share them where wavefronts never exchange
    // data, otherwise the largest of 64 and 32 envs whose rows fit beside the two images
    constexpr int kAcEnvs = S::kWaveLocal ? 512 / S::N : (S::N <= 6 ? 64 : 32);
    const bool ac = mode_is_ac(mode);
    const uint32_t per_block = ac ? uint32_t(kAcEnvs) : 64u;
    if (A.r.TE != A.r.E && A.r.E % per_block != 0) {
      // small runs (the paper's IPPO setting is 16 envs per run): blocks of 16 envs inside a run
      if (A.r.E % 16 == 0)
        return ac ? tag_policy_impl<S, 16, 32, true>(mode, A, packed, packed_critic, s)
                  : tag_policy_impl<S, 16, 32, false>(mode, A, packed, nullptr, s);
      *why = "with several runs, num_envs per run must be a multiple of 16";
      return hipSuccess;
    }
    if constexpr (S::D <= 16) {
      // Small batches (every block has a CU to itself, so the step latency of one block is the time): the
      // rows spread over wavefronts of 32 rows, one per SIMD: 64 envs x 2 agents, 32 envs x 3 or 4 agents.
      // Measured per 128-step rollout up to 8,192 envs of 4 agents: 0.54 against 0.84 ms, bf16 0.36 against
      // 0.59 ms, actor-critic 0.88 against 2.41 ms; two such blocks per CU still win with 2 agents (1.55x)
      // and for the actor-critic rollout of 4 agents (1.4x).
      constexpr int kSmallEnvs = S::N == 2 ? 64 : 32;
      const uint32_t per_cu = (S::N == 2 || (S::N == 4 && ac)) ? 2u : 1u;
      if ((A.r.TE + kSmallEnvs - 1) / kSmallEnvs <= per_cu * compute_units())
        return ac ? tag_policy_impl<S, kSmallEnvs, 32, true>(mode, A, packed, packed_critic, s)
                  : tag_policy_impl<S, kSmallEnvs, 32, false>(mode, A, packed, nullptr, s);
    }
    if (ac) return tag_policy_impl<S, kAcEnvs, 64, true>(mode, A, packed, packed_critic, s);
    return tag_policy_impl<S, 64, 64, false>(mode, A, packed, nullptr, s);
  } else {
    *why = "no policy kernel for this shape (observation rows longer than 32)";
    return hipSuccess;
  }
}

template <typename S>
hipError_t tag_pack(PolicyBuffers& pb, int R, bool bf16, int nout, const float* W1, const float* b1, const float* W2,
                    const float* b2, const float* W3, const float* b3, hipStream_t s) {
  if constexpr (S::D <= 32) {
    using Net = NetShape<S::D, S::D>;
    using P = PkT<false, Net::kWideIn>;
    if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * (bf16 ? PkB::RUN_BYTES : P::RUN_BYTES)); e != hipSuccess)
      return e;
    constexpr int total = pack_threads<Net>();
    if (bf16)
      hipLaunchKernelGGL(pack_bf16_kernel<Net>, dim3((total + 255) / 256, R), dim3(256), 0, s,
                         static_cast<uint8_t*>(pb.packed), W1, b1, W2, b2, W3, b3, nout);
    else
      hipLaunchKernelGGL(pack_split_kernel<Net>, dim3((total + 255) / 256, R), dim3(256), 0, s,
                         static_cast<uint8_t*>(pb.packed), W1, b1, W2, b2, W3, b3, nout);
    return hipGetLastError();
  } else {
    return hipErrorInvalidValue;
  }
}

}  // namespace

// The shapes that are built: (agents, landmarks, good agents).
#define MPE_TAG_SHAPES(X) X(4, 2, 1) X(2, 1, 1) X(3, 0, 1) X(6, 2, 2) X(5, 2, 1) X(8, 2, 2) X(10, 3, 2)

bool tag_supported(int N, int L, int G) {
#define X(n, l, g) if (N == n && L == l && G == g) return true;
  MPE_TAG_SHAPES(X)
#undef X
  return false;
}

bool tag_policy_supported(int N, int L, int G, int H, int weight_dtype) {
  return tag_supported(N, L, G) && H == kH && (weight_dtype == 0 || weight_dtype == 1) &&
         4 + 2 * L + 2 * (N - 1) + 2 * G <= 32;
}

void launch_tag_reset(int N, int L, int G, const StatePtrs& st, uint32_t TE, uint32_t E, uint32_t seed, float* obs,
                      hipStream_t s) {
#define X(n, l, g)                                                                                      \
  if (N == n && L == l && G == g) {                                                                     \
    hipLaunchKernelGGL((tag_reset_kernel<TagShape<n, l, g>>), dim3((TE + 63) / 64), dim3(64 * n), 0, s, st, TE, E, \
                       seed, obs);                                                                      \
    return;                                                                                             \
  }
  MPE_TAG_SHAPES(X)
#undef X
}

hipError_t launch_tag_rollout(int N, int L, int G, int mode, const TagArgs& A, const void* packed,
                              const void* packed_critic, hipStream_t s, const char** why) {
#define X(n, l, g) \
  if (N == n && L == l && G == g) return tag_launch<TagShape<n, l, g>>(mode, A, packed, packed_critic, s, why);
  MPE_TAG_SHAPES(X)
#undef X
  return hipErrorInvalidValue;
}

hipError_t pack_policy_tag(PolicyBuffers& pb, int N, int L, int G, int R, bool bf16, int nout, const float* W1,
                           const float* b1, const float* W2, const float* b2, const float* W3, const float* b3,
                           hipStream_t s) {
#define X(n, l, g) \
  if (N == n && L == l && G == g) return tag_pack<TagShape<n, l, g>>(pb, R, bf16, nout, W1, b1, W2, b2, W3, b3, s);
  MPE_TAG_SHAPES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace mpe
