// Fused rollout kernel for the headline shape: fp32 policy 6N -> 64 -> 64 -> 5 (N <= 3 agents; with fp32 weights
// also 4 to 10 agents, whose 4N + 2 live inputs fill one K slice of layer 1 (up to 7 agents, 64-env blocks) or two
// (8 to 10 agents, 32-env blocks)),
// shared by all agents or one set of weights per run (paper: App. G IPPO table, two tanh layers
// of width 64; Sec. 3.2 parameter sharing; Sec. 5.2 and App. E: whole training runs vectorised on one device).
//
// Where the contraction runs.  On gfx950 the fp32 MFMA shares the vector datapath: fp32 matrix
// and fp32 vector peaks are the same number, and measured MFMA-f32 and VALU time add up instead
// of overlapping.  The 16-bit matrix cores are a separate unit, 16x faster per K.  So every fp32
// operand is split into three fp16 terms
//     x = h + m + l,   h = x truncated to fp16, m = (x - h) truncated, l = x - h - m truncated
// (11 + 11 + 2 = 24 significant bits, each difference exact in fp32: the split is exact for
// 0.5 <= |x| < 65,504 and within 2^-24 absolute below, see mpe_mlp64.h) and the product of two
// operands is accumulated in fp32 from the six cross terms of weight >= 2^-22:
//     x*w ~= hh + hm + mh + mm + hl + lh      (dropped: ml + lm + ll <= 2^-32 |x w|)
// i.e. the operand values of an fp32 GEMM to within half an fp32 rounding of a number of size 1.
// Weights are split once by the pack kernel; activations are split in registers (7 vector
// instructions per pair of values; the earlier split into three bf16 terms, 8 + 8 + 8 bits, exact
// everywhere, took 11 and made the whole rollout 4-5 % slower).
//
// Mapping: one lane per agent row; a wavefront owns 64 rows = two pairs of 16-row tiles; each
// A operand (weights, from LDS) is loaded once per pair.  The accumulator layout of
// v_mfma_f32_16x16x32_f16 / _bf16 (lane (j, gq) holds batch row j and hidden units 16m + 4gq + r) is
// again a B-operand layout for the next layer when the weights are packed in the matching K
// order, so activations stay in registers between layers.  Every wavefront works on its own
// rows of the LDS observation tile; the only cross-wavefront data are the new positions of the
// envs that straddle a wavefront boundary: one barrier per step among the N wavefronts of a
// 64-env sync group (the block barrier for 64-env blocks, an arrival counter in LDS for the
// 256-env blocks of four independent groups).
//
// The same kernel also serves the mixed per-agent reward (PER_AGENT), the actor-critic rollout
// (AC: a second pass of the tile code over a critic's packed image, log-probability of the
// sampled action) and the bf16 variant of the same shapes (BF: weights and layer inputs rounded
// to bf16, nearest even, fp32 accumulation -- one matrix instruction per product instead of
// six, no operand split; policy_pair_bf).
#include "mpe_mlp64.h"

namespace mpe {

namespace {

// simple spread: rows of 6N floats, of which the first 4N + 2 are not always zero
template <int N>
using SpreadNet = NetShape<6 * N, 4 * N + 2>;

// Plain rollout: W1A + W2A and the biases of the policy (its W3A lives in registers).
// Actor-critic rollout (AC): the whole packed image of the policy and of the critic (W1A, W2A,
// W3A, biases each), a value per row, and one arrival counter per 64-env sync group.
// ROWS = the block's agent rows, rounded up to whole wavefronts of RW rows (only 16-env blocks of
// 3 agents have such padding rows: 48 -> 64; no env owns them and nothing of them leaves the block).
template <int N, int EB, bool AC = false, bool BF = false, int RW = 64>
struct SmemF32 {
  using P = PkT<BF, SpreadNet<N>::kWideIn, SpreadNet<N>::kSlices1>;
  static constexpr int D = 6 * N;
  static constexpr int ROWS = (EB * N + RW - 1) / RW * RW;
  // LEAN (actor-critic in 16-env blocks, i.e. many small runs): W3A of both networks stays in global memory
  // (re-read every step, 64 bytes per lane), so that two blocks fit a CU instead of one.
  static constexpr bool LEAN = AC && EB == 16;
  static constexpr size_t OFF_BIAS = (AC && !LEAN) ? P::OFF_BIAS : P::LDS_BYTES;
  static constexpr size_t OFF_CRITIC = OFF_BIAS + P::BIAS_BYTES;     // AC: the critic's packed image
  static constexpr size_t CRITIC_BIAS = LEAN ? P::LDS_BYTES : P::OFF_BIAS;   // offset of its biases inside it
  static constexpr size_t OFF_OBS = OFF_CRITIC + (AC ? (LEAN ? P::LDS_BYTES + P::BIAS_BYTES : P::RUN_BYTES) : 0);
  static constexpr size_t OBS = size_t(ROWS) * D * 4 + 64;           // + zeroed tail: layer 1 reads 16 cols
  static constexpr size_t OFF_NEWPOS = OFF_OBS + OBS;                // [2][ROWS] float2, by step parity
  static constexpr size_t OFF_VALUE = OFF_NEWPOS + size_t(2) * ROWS * 8;   // AC: [ROWS] float
  static constexpr size_t OFF_ARRIVED = OFF_VALUE + (AC ? size_t(ROWS) * 4 : 0);
  static constexpr size_t TOTAL = OFF_ARRIVED + (EB > 64 ? 16 : 0);
  static_assert(OFF_OBS % 16 == 0 && OFF_NEWPOS % 16 == 0 && OFF_CRITIC % 16 == 0 && EB / 64 <= 4, "alignment");
};

// PER_AGENT: rew_traj is [T][TE][N], the mixed per-agent reward; every lane stores its agent's.
// AC (actor-critic outputs): a second network of the same shape with one output, `packed_critic`,
// is evaluated on every observation acted on, and the log-probability of the sampled action is
// recorded (paper Sec. 3.2: IPPO / MAPPO; App. G: two tanh layers of width 64).  A block is then
// EB / 64 independent 64-env sync groups that share the two staged networks.
//
// RW = rows per wavefront.  64: one lane per row.  32 (64-env blocks only, for batches that leave CUs
// empty): twice the wavefronts, each with ONE pair of 16-row tiles; lanes 32..63 are exact clones of
// lanes 0..31 (same row, same inputs, same arithmetic, so their LDS writes repeat the same values)
// that store nothing to global memory.  The step latency of a block, which is all that matters when
// every block has a CU to itself, is then one pair of tiles plus the env step instead of two pairs.
template <int N, int EB, int MINW, bool PER_AGENT, bool AC, bool BF, int RW = 64>
__global__ __launch_bounds__((EB * N + RW - 1) / RW * 64, MINW) void rollout_policy_f32_kernel(RolloutArgs A, const uint8_t* __restrict__ packed,
                                                                          const uint8_t* __restrict__ packed_critic,
                                                                          int per_run_weights, uint32_t groups,
                                                                          uint32_t groups_per_xcd) {
  using M = SmemF32<N, EB, AC, BF, RW>;
  using P = typename M::P;

  constexpr int D = 6 * N, ROWS = M::ROWS, THREADS = ROWS * (64 / RW);
  constexpr bool kPadded = ROWS != EB * N;
  static_assert(THREADS % 64 == 0, "block must be whole wavefronts");
  static_assert(RW == 64 || (RW == 32 && EB <= 64), "half-filled wavefronts only in blocks of one sync group");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* wsm = smem;
  float* bias = reinterpret_cast<float*>(smem + M::OFF_BIAS);
  float* tile = reinterpret_cast<float*>(smem + M::OFF_OBS);
  float2* newpos = reinterpret_cast<float2*>(smem + M::OFF_NEWPOS);
  const uint8_t* csm = smem + M::OFF_CRITIC;                                         // AC only
  const float* cbias = reinterpret_cast<const float*>(smem + M::OFF_CRITIC + M::CRITIC_BIAS);
  float* values = reinterpret_cast<float*>(smem + M::OFF_VALUE);

  // Wavefront -> rows.  With several sync groups per block (EB > 64) the N wavefronts of group g are
  // the hardware wavefronts g, g + G, g + 2G (G = EB / 64 groups): the hardware deals the wavefronts
  // of a block to the four SIMDs in turn, so with G = 4 a group's wavefronts share ONE SIMD, and a
  // wavefront waiting at the group's per-step barrier yields its issue slots to the very wavefronts
  // it is waiting for (measured at 65,536 envs x 128 steps: 2.06 ms per rollout against 2.30 ms with the
  // wavefronts of a group dealt to three different SIMDs).
  // `wave` and `tid` below are these virtual indices: row = tid.
  const int lane = threadIdx.x & 63;
  const int hw_wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  constexpr int kGroups = EB > 64 ? EB / 64 : 1;
  const int wave = kGroups > 1 ? (hw_wave % kGroups) * N + hw_wave / kGroups : hw_wave;
  const int tid = wave * RW + (lane & (RW - 1));     // this lane's row
  const int el_row = tid / N, i = tid - el_row * N;  // env within block, agent
  const bool in_block = !kPadded || el_row < EB;     // false for padding rows: they shadow env 0 of the block
  const int el = in_block ? el_row : 0;
  const size_t TE = A.TE;
  // XCD-aware mapping: the hardware deals block b to XCD b % 8; giving each XCD one contiguous
  // range of env groups lets the partial cache lines that neighbouring groups write per step
  // (actions 3*EB bytes, done EB bytes) merge in one L2 instead of being written back apart.
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
  const int nvalid = left < size_t(EB) ? int(left) : EB;   // valid envs in this block
  // rows of this wavefront that belong to valid envs
  const int wave_rows = min(max(nvalid * N - wave * RW, 0), RW);

  // ---- stage this block's weights (the run of its first env): W1A, W2A, biases in LDS; W3A in registers
  const uint8_t* run_weights = packed + (per_run_weights ? size_t(uint32_t(g0) / A.E) * P::RUN_BYTES : 0);
  [[maybe_unused]] const uint8_t* critic_weights =
      AC ? packed_critic + (per_run_weights ? size_t(uint32_t(g0) / A.E) * P::RUN_BYTES : 0) : nullptr;
  // where the layer-3 operands are re-read from in the actor-critic rollout
  [[maybe_unused]] const uint8_t* w3_policy = M::LEAN ? run_weights : smem;
  [[maybe_unused]] const uint8_t* w3_critic = M::LEAN ? critic_weights : smem + M::OFF_CRITIC;
  // A operands of layer 3 from a packed image (global memory or LDS)
  auto load_w3 = [&](const uint8_t* image) {
    W3Terms w;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if constexpr (BF || SpreadNet<N>::kRowTerms) {
        w.s[s].h = reinterpret_cast<const bf16x8*>(image + P::OFF_W3A)[s * 64 + lane];
      } else {
        const bf16x8* src = reinterpret_cast<const bf16x8*>(image + P::OFF_W3A) + s * 3 * 64 + lane;
        w.s[s].h = src[0];
        w.s[s].m = src[64];
        w.s[s].l = src[128];
      }
    }
    return w;
  };
  W3Terms w3;
  if constexpr (!AC) w3 = load_w3(run_weights);
  {
    // the packed image is W1A, W2A, W3A, biases; plain rollouts skip W3A (it is in registers)
    const uint4* src = reinterpret_cast<const uint4*>(run_weights);
    uint4* dst = reinterpret_cast<uint4*>(wsm);
    if constexpr (M::LEAN) {
      // W1A + W2A and the biases of both networks
      const uint4* csrc = reinterpret_cast<const uint4*>(critic_weights);
      uint4* cdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC);
      for (int k = threadIdx.x; k < int(P::LDS_BYTES / 16); k += THREADS) {
        dst[k] = src[k];
        cdst[k] = csrc[k];
      }
      const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + P::OFF_BIAS);
      const uint4* cbsrc = reinterpret_cast<const uint4*>(critic_weights + P::OFF_BIAS);
      uint4* bdst = reinterpret_cast<uint4*>(bias);
      uint4* cbdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC + M::CRITIC_BIAS);
      for (int k = threadIdx.x; k < int(P::BIAS_BYTES / 16); k += THREADS) {
        bdst[k] = bsrc[k];
        cbdst[k] = cbsrc[k];
      }
    } else if constexpr (AC) {
      for (int k = threadIdx.x; k < int(P::RUN_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* csrc = reinterpret_cast<const uint4*>(critic_weights);
      uint4* cdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC);
      for (int k = threadIdx.x; k < int(P::RUN_BYTES / 16); k += THREADS) cdst[k] = csrc[k];
    } else {
      for (int k = threadIdx.x; k < int(P::LDS_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + P::OFF_BIAS);
      uint4* bdst = reinterpret_cast<uint4*>(bias);
      for (int k = threadIdx.x; k < int(P::BIAS_BYTES / 16); k += THREADS) bdst[k] = bsrc[k];
    }
    if (threadIdx.x < 16) tile[ROWS * D + threadIdx.x] = 0.0f;
    if constexpr (EB > 64) {
      if (threadIdx.x < EB / 64) reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED)[threadIdx.x] = 0u;
    }
  }

  // ---- registers: own agent, all agents' positions, all landmarks
  float px = 0.0f, py = 0.0f, vx = 0.0f, vy = 0.0f;
  float qx[N], qy[N], lx[N], ly[N];
  int32_t ep = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) qx[a] = qy[a] = lx[a] = ly[a] = 0.0f;
  if (in_range) {
#pragma unroll
    for (int a = 0; a < N; ++a) {
      qx[a] = A.st.pos_a[(0 * N + a) * TE + g];
      qy[a] = A.st.pos_a[(1 * N + a) * TE + g];
      lx[a] = A.st.pos_l[(0 * N + a) * TE + g];
      ly[a] = A.st.pos_l[(1 * N + a) * TE + g];
    }
    vx = A.st.vel_a[(0 * N + i) * TE + g];
    vy = A.st.vel_a[(1 * N + i) * TE + g];
    ep = A.st.ep_step[g];
  }
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a == i) { px = qx[a]; py = qy[a]; }
  }

  // Write this lane's observation row into the tile (the zero comm slots only the first time).
  auto write_obs_row = [&](bool with_zeros) {
    float2* row = reinterpret_cast<float2*>(tile + tid * D);
    int c = 0;
    row[c++] = make_float2(vx, vy);
    row[c++] = make_float2(px, py);
#pragma unroll
    for (int l = 0; l < N; ++l) row[c++] = make_float2(lx[l] - px, ly[l] - py);
#pragma unroll
    for (int a = 0; a < N; ++a) {
      if (a != i) row[c++] = make_float2(qx[a] - px, qy[a] - py);
    }
    if (with_zeros) {
      for (int zc = 0; zc < N - 1; ++zc) row[c + zc] = make_float2(0.0f, 0.0f);
    }
  };
  write_obs_row(true);
  __syncthreads();  // weights, biases, zero tail staged; from here on wavefronts only meet at (C)

  // Output addresses = uniform per-step base (advanced once per step, lives in SGPRs) + a
  // 32-bit lane offset that never changes.
  const size_t wave_row0 = (g0 * N + size_t(wave) * RW) * D;   // float offset of this wavefront's rows in a slice
  float* obs_p = A.obs_traj ? A.obs_traj + wave_row0 : nullptr;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  float* logp_base = A.logp_traj;
  float* value_base = A.value_traj;
  const size_t row_off = size_t(gc) * N + i;          // index of this agent inside a time slice
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  uint32_t step = A.abs_step;
  const float* wtile = tile + wave * (RW * D);        // this wavefront's rows
  uint32_t* arrived = reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED) + wave / N;   // EB > 64 only

  // Critic forward of this wavefront's rows: values[row] (wave-local rows).
  auto critic_rows = [&]() {
#pragma unroll 1
    for (int pr = 0; pr < RW / 32; ++pr) {
      float* rows = tile + (wave * RW + pr * 32) * D;
      float* vals = values + wave * RW + pr * 32;
      const W3Terms wc = load_w3(w3_critic);
      if constexpr (BF) policy_pair_bf<SpreadNet<N>, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
      else policy_pair<SpreadNet<N>, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
    }
  };

  // Stream this wavefront's rows of the tile to dst (its slot in a [env][N][D] slice).
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
    // ---- critic first (it leaves the rows untouched), then the policy, whose logits replace the
    // first columns of the rows: two pairs of 16-row tiles per wavefront each
    if constexpr (AC) critic_rows();
#pragma unroll 1
    for (int pr = 0; pr < RW / 32; ++pr) {
      float* rows = tile + (wave * RW + pr * 32) * D;
      if constexpr (AC) w3 = load_w3(w3_policy);
      if constexpr (BF) policy_pair_bf<SpreadNet<N>>(wsm, bias, w3, rows, rows + 16 * D, lane);
      else policy_pair<SpreadNet<N>>(wsm, bias, w3, rows, rows + 16 * D, lane);
    }
    wave_sync();
    float z[kNumActions];
#pragma unroll
    for (int k = 0; k < kNumActions; ++k) z[k] = tile[tid * D + k];
    if constexpr (!BF && SpreadNet<N>::kRowTerms) z[4] = (z[4] + tile[tid * D + 5]) + tile[tid * D + 6];
    const uint32_t act = gumbel_argmax(z, A.seed, run, env, step, uint32_t(i));
    if (act_base) {
      if (valid) act_base[row_off] = uint8_t(act);
      act_base += TE * N;
    }
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

    // ---- transition of this lane's agent
    agent_move<N>(act, i, A.ph, px, py, vx, vy, qx, qy);
    float2* np = newpos + (t & 1) * ROWS;
    np[tid] = make_float2(px, py);
    // (C) new positions of every agent of every env of this 64-env group are visible
    if constexpr (EB <= 64) __syncthreads();
    else if constexpr (N > 1) group_barrier(arrived, uint32_t(N) * uint32_t(t + 1), lane, A.fault, A.barrier_polls);
    else wave_sync();

#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float2 p = np[el * N + a];
      qx[a] = p.x;
      qy[a] = p.y;
    }
    // shared coverage reward, evaluated by every lane (N*N distances), stored by agent 0
    {
      const float r = coverage_reward(qx, qy, lx, ly);
      if constexpr (PER_AGENT) {
        const uint32_t overlaps = overlap_count<N>(i, px, py, qx, qy, A.ph);
        if (rew_base) {
          if (valid) rew_base[row_off] = mixed_reward(r, overlaps, A.ph);
          rew_base += TE * N;
        }
      } else if (rew_base) {
        if (env_writer) rew_base[gc] = r;
        rew_base += TE;
      }
    }
    ep += 1;
    const bool done = ep >= A.ph.max_ep;
    if (done_base) {
      if (env_writer) done_base[gc] = done ? 1 : 0;
      done_base += TE;
    }
    if (done) {
      // new episode keyed by step + 1; every lane regenerates the whole env (rare: 1 step in
      // max_ep).  The empty asm keeps the compiler from hoisting the env-dependent first Philox
      // round of all 2N streams out of the step loop, where it would only cost registers.
      uint32_t env_r = env;
      asm volatile("" : "+v"(env_r));
#pragma unroll
      for (int a = 0; a < N; ++a) {
        const uint4 w = philox4x32_10(env_r, step + 1u, uint32_t(a), kTagResetPos, A.seed, run);
        qx[a] = word_to_position(w.x);
        qy[a] = word_to_position(w.y);
        const uint4 wl = philox4x32_10(env_r, step + 1u, uint32_t(N + a), kTagResetPos, A.seed, run);
        lx[a] = word_to_position(wl.x);
        ly[a] = word_to_position(wl.y);
      }
#pragma unroll
      for (int a = 0; a < N; ++a) {
        if (a == i) { px = qx[a]; py = qy[a]; }
      }
      vx = vy = 0.0f;
      ep = 0;
    }
    write_obs_row(false);
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
#pragma unroll
    for (int l = 0; l < N; ++l) {
      if (l == i) {
        A.st.pos_l[(0 * N + l) * TE + g] = lx[l];
        A.st.pos_l[(1 * N + l) * TE + g] = ly[l];
      }
    }
    if (i == 0) A.st.ep_step[g] = ep;
  }
}

// --------------------------------------------------------------------------------------
// Per-run weights at full occupancy.  A block is 256 envs = four 64-env sync groups, EACH WITH THE
// WEIGHTS OF ITS OWN RUN in LDS (4 x 33 KB), the wavefronts of a group on one SIMD as above.  That
// leaves no room for observation tiles, so a lane keeps its row in registers and stores it to the
// trajectory itself, and the layer-1 operands and the logits travel between the row's lane and the
// matrix layout by 4 x 4 lane-group transposes (permlane swaps, no memory).  Same arithmetic, in
// the same order, as the kernel above: results are bit-identical.  fp32 weights, either reward,
// N = 2 or 3 (layer 3 in the row-term layout), runs of a multiple of 64 envs.
// --------------------------------------------------------------------------------------
template <int N>
struct SmemReg {
  static constexpr int G = 4, ROWS_G = 64 * N;                         // groups per block, rows per group
  static constexpr size_t GROUP_W = Pk::LDS_BYTES + Pk::BIAS_BYTES;    // W1A, W2A, then the biases
  static constexpr size_t OFF_NEWPOS = G * GROUP_W;                    // [G][2][ROWS_G] float2, by step parity
  static constexpr size_t OFF_ARRIVED = OFF_NEWPOS + size_t(G) * 2 * ROWS_G * 8;
  static constexpr size_t TOTAL = OFF_ARRIVED + 16;
  static_assert(GROUP_W % 16 == 0 && TOTAL <= 160 * 1024, "LDS");
};

template <int N, bool PER_AGENT>
__global__ __launch_bounds__(256 * N, 1) void rollout_policy_f32_reg_kernel(RolloutArgs A, const uint8_t* __restrict__ packed,
                                                                            uint32_t blocks, uint32_t blocks_per_xcd) {
  using M = SmemReg<N>;
  using Net = SpreadNet<N>;
  static_assert(Net::kRowTerms, "layer 3 in the row-term layout");
  constexpr int D = 6 * N, KIN = Net::KIN, ROWS_G = M::ROWS_G;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int lane = threadIdx.x & 63;
  const int hw_wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  const int gi = hw_wave & 3;                 // sync group: hardware wavefronts gi, gi + 4, gi + 8 share a SIMD
  const int r = (hw_wave >> 2) * 64 + lane;   // row inside the group
  const int el = r / N, i = r - el * N;       // env within the group, agent
  const size_t TE = A.TE;
  const uint32_t blk = (blockIdx.x & 7u) * blocks_per_xcd + (blockIdx.x >> 3);
  if (blk >= blocks) return;  // whole block, before any barrier
  const size_t gg0 = size_t(blk) * 256 + size_t(gi) * 64;   // first env of this group
  const size_t g = gg0 + el;
  const bool valid = g < TE;
  const uint32_t gc = valid ? uint32_t(g) : uint32_t(blk) * 256u;   // a block has at least one env
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;

  // ---- this group's weights (the run of its first env; runs are multiples of 64 envs)
  uint8_t* wsm = smem + size_t(gi) * M::GROUP_W;
  const float* bias = reinterpret_cast<const float*>(wsm + Pk::LDS_BYTES);
  const uint32_t grun = uint32_t(gg0 < TE ? gg0 : size_t(blk) * 256) / A.E;
  const uint8_t* run_weights = packed + size_t(grun) * Pk::RUN_BYTES;
  W3Terms w3;
#pragma unroll
  for (int s = 0; s < 2; ++s) w3.s[s].h = reinterpret_cast<const bf16x8*>(run_weights + Pk::OFF_W3A)[s * 64 + lane];
  {
    const uint4* src = reinterpret_cast<const uint4*>(run_weights);
    uint4* dst = reinterpret_cast<uint4*>(wsm);
    for (int k = r; k < int(Pk::LDS_BYTES / 16); k += ROWS_G) dst[k] = src[k];
    const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + Pk::OFF_BIAS);
    uint4* bdst = reinterpret_cast<uint4*>(wsm + Pk::LDS_BYTES);
    for (int k = r; k < int(Pk::BIAS_BYTES / 16); k += ROWS_G) bdst[k] = bsrc[k];
    if (threadIdx.x < 4) reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED)[threadIdx.x] = 0u;
  }
  float2* newpos = reinterpret_cast<float2*>(smem + M::OFF_NEWPOS) + size_t(gi) * 2 * ROWS_G;
  uint32_t* arrived = reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED) + gi;

  // ---- registers: own agent, all agents' positions, all landmarks
  float px = 0.0f, py = 0.0f, vx = 0.0f, vy = 0.0f;
  float qx[N], qy[N], lx[N], ly[N];
  int32_t ep = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) qx[a] = qy[a] = lx[a] = ly[a] = 0.0f;
  if (valid) {
#pragma unroll
    for (int a = 0; a < N; ++a) {
      qx[a] = A.st.pos_a[(0 * N + a) * TE + g];
      qy[a] = A.st.pos_a[(1 * N + a) * TE + g];
      lx[a] = A.st.pos_l[(0 * N + a) * TE + g];
      ly[a] = A.st.pos_l[(1 * N + a) * TE + g];
    }
    vx = A.st.vel_a[(0 * N + i) * TE + g];
    vy = A.st.vel_a[(1 * N + i) * TE + g];
    ep = A.st.ep_step[g];
  }
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a == i) { px = qx[a]; py = qy[a]; }
  }

  // This lane's observation row: the KIN leading entries (the rest of the row is zero).
  float o[16];
  auto build_row = [&]() {
#pragma unroll
    for (int c = 0; c < 16; ++c) o[c] = 0.0f;
    o[0] = vx; o[1] = vy; o[2] = px; o[3] = py;
#pragma unroll
    for (int l = 0; l < N; ++l) { o[4 + 2 * l] = lx[l] - px; o[5 + 2 * l] = ly[l] - py; }
    // the k-th OTHER agent is agent k (k < i) or k + 1
#pragma unroll
    for (int k = 0; k < N - 1; ++k) {
      const bool up = k >= i;
      o[4 + 2 * N + 2 * k] = (up ? qx[k + 1] : qx[k]) - px;
      o[5 + 2 * N + 2 * k] = (up ? qy[k + 1] : qy[k]) - py;
    }
  };
  auto store_row = [&](float* dst) {   // dst: this lane's row of a [TE][N][D] slice
    float2* d2 = reinterpret_cast<float2*>(dst);
#pragma unroll
    for (int c = 0; c < KIN / 2; ++c) d2[c] = make_float2(o[2 * c], o[2 * c + 1]);
#pragma unroll
    for (int c = KIN / 2; c < D / 2; ++c) d2[c] = make_float2(0.0f, 0.0f);
  };
  build_row();
  __syncthreads();  // weights and biases staged, counters cleared; from here on wavefronts only meet at (C)

  const size_t row_off = size_t(gc) * N + i;          // index of this agent inside a time slice
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  float* obs_base = A.obs_traj;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  uint32_t step = A.abs_step;

  for (int t = 0; t < A.T; ++t, ++step) {
    if (obs_base) {
      if (valid) store_row(obs_base + row_off * D);
      obs_base += TE * (N * D);
    }
    // ---- policy: the rows of tile c belong to lane group c; lane (j, gq) needs inputs 8 (gq & 1) .. + 7
    // of row 16 c + j: the transpose of {low, high, low, high} halves of the row between register index
    // and lane group
    f32x4 z[4];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      float inX[1][8], inY[1][8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint32_t v[4] = {__float_as_uint(o[e]), __float_as_uint(o[8 + e]), __float_as_uint(o[e]), __float_as_uint(o[8 + e])};
        transpose_groups(v);
        inX[0][e] = __uint_as_float(v[2 * pr]);
        inY[0][e] = __uint_as_float(v[2 * pr + 1]);
      }
      policy_core<Net>(wsm, bias, w3, inX, inY, z[2 * pr], z[2 * pr + 1], lane);
    }
    // ---- logits back to the row's lane: lane (j, gq) holds, for tile c, output gq (sum of its three
    // term rows) and term gq of output 4
    float zz[kNumActions];
    {
      uint32_t sv[4], tv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        sv[c] = __float_as_uint((z[c][0] + z[c][1]) + z[c][2]);
        tv[c] = __float_as_uint(z[c][3]);
      }
      transpose_groups(sv);
      transpose_groups(tv);
#pragma unroll
      for (int k = 0; k < 4; ++k) zz[k] = __uint_as_float(sv[k]);
      zz[4] = (__uint_as_float(tv[0]) + __uint_as_float(tv[1])) + __uint_as_float(tv[2]);
    }
    const uint32_t act = gumbel_argmax(zz, A.seed, run, env, step, uint32_t(i));
    if (act_base) {
      if (valid) act_base[row_off] = uint8_t(act);
      act_base += TE * N;
    }

    // ---- transition of this lane's agent
    agent_move<N>(act, i, A.ph, px, py, vx, vy, qx, qy);
    float2* np = newpos + (t & 1) * ROWS_G;
    np[r] = make_float2(px, py);
    // (C) new positions of every agent of every env of this 64-env group are visible
    group_barrier(arrived, uint32_t(N) * uint32_t(t + 1), lane, A.fault, A.barrier_polls);
#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float2 p = np[el * N + a];
      qx[a] = p.x;
      qy[a] = p.y;
    }
    // shared coverage reward, evaluated by every lane (N*N distances), stored by agent 0
    {
      const float rw = coverage_reward(qx, qy, lx, ly);
      if constexpr (PER_AGENT) {
        const uint32_t overlaps = overlap_count<N>(i, px, py, qx, qy, A.ph);
        if (rew_base) {
          if (valid) rew_base[row_off] = mixed_reward(rw, overlaps, A.ph);
          rew_base += TE * N;
        }
      } else if (rew_base) {
        if (env_writer) rew_base[gc] = rw;
        rew_base += TE;
      }
    }
    ep += 1;
    const bool done = ep >= A.ph.max_ep;
    if (done_base) {
      if (env_writer) done_base[gc] = done ? 1 : 0;
      done_base += TE;
    }
    if (done) {
      // new episode keyed by step + 1; every lane regenerates the whole env (1 step in max_ep)
      uint32_t env_r = env;
      asm volatile("" : "+v"(env_r));
#pragma unroll
      for (int a = 0; a < N; ++a) {
        const uint4 w = philox4x32_10(env_r, step + 1u, uint32_t(a), kTagResetPos, A.seed, run);
        qx[a] = word_to_position(w.x);
        qy[a] = word_to_position(w.y);
        const uint4 wl = philox4x32_10(env_r, step + 1u, uint32_t(N + a), kTagResetPos, A.seed, run);
        lx[a] = word_to_position(wl.x);
        ly[a] = word_to_position(wl.y);
      }
#pragma unroll
      for (int a = 0; a < N; ++a) {
        if (a == i) { px = qx[a]; py = qy[a]; }
      }
      vx = vy = 0.0f;
      ep = 0;
    }
    build_row();
  }
  if (A.last_obs && valid) store_row(A.last_obs + row_off * D);

  // ---- state back to HBM
  if (valid) {
    A.st.pos_a[(0 * N + i) * TE + g] = px;
    A.st.pos_a[(1 * N + i) * TE + g] = py;
    A.st.vel_a[(0 * N + i) * TE + g] = vx;
    A.st.vel_a[(1 * N + i) * TE + g] = vy;
#pragma unroll
    for (int l = 0; l < N; ++l) {
      if (l == i) {
        A.st.pos_l[(0 * N + l) * TE + g] = lx[l];
        A.st.pos_l[(1 * N + l) * TE + g] = ly[l];
      }
    }
    if (i == 0) A.st.ep_step[g] = ep;
  }
}

template <int N, bool PER_AGENT>
hipError_t rollout_reg_impl(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s) {
  using M = SmemReg<N>;
  auto kern = rollout_policy_f32_reg_kernel<N, PER_AGENT>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (hipError_t e = allow_lds(reinterpret_cast<const void*>(kern), M::TOTAL, lds_allowed); e != hipSuccess) return e;
  const uint32_t blocks = (A.TE + 255) / 256;
  const uint32_t per_xcd = (blocks + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(256 * N), M::TOTAL, s, A, static_cast<const uint8_t*>(pb.packed),
                     blocks, per_xcd);
  return hipGetLastError();
}

template <int N, int EB, int MINW, bool PER_AGENT, bool AC, bool BF, int RW = 64>
hipError_t rollout_impl(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const void* critic = nullptr) {
  using M = SmemF32<N, EB, AC, BF, RW>;
  auto kern = rollout_policy_f32_kernel<N, EB, MINW, PER_AGENT, AC, BF, RW>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (hipError_t e = allow_lds(reinterpret_cast<const void*>(kern), M::TOTAL, lds_allowed); e != hipSuccess) return e;
  const uint32_t groups = (A.TE + EB - 1) / EB;
  const uint32_t per_xcd = (groups + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(M::ROWS * (64 / RW)), M::TOTAL, s, A,
                     static_cast<const uint8_t*>(pb.packed), static_cast<const uint8_t*>(critic), int(A.TE != A.E), groups,
                     per_xcd);
  return hipGetLastError();
}

template <int N>
hipError_t pack_impl(PolicyBuffers& pb, int R, const float* W1, const float* b1, const float* W2,
                     const float* b2, const float* W3, const float* b3, int nout, bool bf16, hipStream_t s) {
  const size_t run_bytes = PkT<false, SpreadNet<N>::kWideIn, SpreadNet<N>::kSlices1>::RUN_BYTES;
  if (bf16 && N > 3) return hipErrorInvalidValue;
  const size_t bytes1 = bf16 ? PkB::RUN_BYTES : run_bytes;
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * bytes1); e != hipSuccess) return e;
  constexpr int total = pack_threads<SpreadNet<N>>();
  dim3 grid((total + 255) / 256, R);
  if constexpr (N <= 3) {
    if (bf16) {
      hipLaunchKernelGGL(pack_bf16_kernel<SpreadNet<N>>, grid, dim3(256), 0, s, static_cast<uint8_t*>(pb.packed), W1, b1, W2,
                         b2, W3, b3, nout);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL(pack_split_kernel<SpreadNet<N>>, grid, dim3(256), 0, s, static_cast<uint8_t*>(pb.packed), W1, b1, W2,
                     b2, W3, b3, nout);
  return hipGetLastError();
}

// Small batches: when every block has a CU (nearly) to itself, the time of a rollout is the step latency of
// one block (one wavefront per SIMD running its matrix and vector instructions back to back), so the rows
// are spread over more wavefronts of 32 rows = one pair of 16-row tiles each, one wavefront per SIMD where
// that works out.  Measured per 128-step rollout, against N wavefronts of 64 rows:
//   64 envs x 1 or 2 agents = 2 or 4 wavefronts: 0.48 / 0.50 ms against 0.76 / 0.77 ms up to one block per
//     CU, still 1.07x / 1.18x at three blocks per CU (the most that are resident);
//   32 envs x 3 agents = 3 wavefronts, while such blocks have a CU each (8,192 envs): 0.51 against 0.81 ms
//     (actor-critic 0.85 against 1.51 ms);
//   64 envs x 3 agents = 6 wavefronts, two SIMDs with two: 0.73 against 0.82 ms up to one block per CU,
//     slower beyond.
enum SmallShape { kRegular = 0, kHalf64 = 1, kHalf32 = 2 };
template <int N>
SmallShape small_shape(const RolloutArgs& A) {
  const uint32_t cus = compute_units();
  if (N == 3 && (A.TE + 31) / 32 <= cus) return kHalf32;
  if ((A.TE + 63) / 64 <= (N == 3 ? cus : 4 * cus)) return kHalf64;
  return kRegular;
}

template <int N, bool PER_AGENT, bool AC, bool BF>
hipError_t launch_blocks64(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const void* critic) {
  const SmallShape shape = small_shape<N>(A);
  if constexpr (N == 3) {
    if (shape == kHalf32) return rollout_impl<N, 32, 1, PER_AGENT, AC, BF, 32>(A, pb, s, critic);
  }
  if (shape == kHalf64) return rollout_impl<N, 64, 1, PER_AGENT, AC, BF, 32>(A, pb, s, critic);
  return rollout_impl<N, 64, 3, PER_AGENT, AC, BF>(A, pb, s, critic);
}

// Envs per block.  64 (N wavefronts, one block barrier per step) is the general shape: three
// blocks are resident per CU, and with several runs every block must lie inside one run.  When
// one run has at least one 256-env block per CU, blocks of 256 envs = four independent 64-env
// sync groups (12 wavefronts, per-group arrival counters) fill the chip in whole rounds with no
// tail of single resident blocks: measured 2.06 ms against 2.37 ms at 65,536 envs x 3 agents.
// (Two 128-env blocks per CU with ONE block barrier among six wavefronts were slower: 2.97 ms.)
template <int N, bool BF>
hipError_t launch_n(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const char** why) {
  const bool one_run = A.TE == A.E;
  const bool per_agent = A.ph.reward_mode == 1;
  if constexpr (N > 3) {
    // 4 to 10 agents (fp32 weights; bf16 ones run the lane-per-agent bf16 kernel): blocks of 64 envs (N wavefronts,
    // one or two per CU by their LDS) up to 7 agents, of 32 envs beyond (the rows are 6 N floats wide)
    static_assert(!BF, "bf16 weights with 4 and more agents are another kernel's");
    constexpr int kEnvs = N <= 7 ? 64 : 32;
    if (!one_run && A.E % kEnvs != 0) {
      *why = "with several runs and 4 or more agents, num_envs per run must be a multiple of 64 (of 32 with 8 to 10 agents)";
      return hipSuccess;
    }
    return per_agent ? rollout_impl<N, kEnvs, 1, true, false, false>(A, pb, s) : rollout_impl<N, kEnvs, 1, false, false, false>(A, pb, s);
  } else {
  if (one_run && A.TE / 256 >= compute_units())
    return per_agent ? rollout_impl<N, 256, 3, true, false, BF>(A, pb, s) : rollout_impl<N, 256, 3, false, false, BF>(A, pb, s);
  if constexpr (!BF && N >= 2) {
    // several runs that fill the chip in (nearly) whole rounds of one block per CU: 256-env blocks of four
    // groups, each with its own run's weights (1,024 runs x 64 envs x 3 agents: 2.04 ms against 2.44 ms
    // with 64-env blocks; with a tail round that is mostly empty the 64-env blocks are faster)
    if (!one_run && A.E % 64 == 0) {
      const uint32_t blocks = (A.TE + 255) / 256, cus = compute_units();
      const uint32_t rounds = (blocks + cus - 1) / cus;
      if (blocks >= cus && uint64_t(blocks) * 10 >= uint64_t(rounds) * cus * 9)
        return per_agent ? rollout_reg_impl<N, true>(A, pb, s) : rollout_reg_impl<N, false>(A, pb, s);
    }
  }
  if (one_run || A.E % 64 == 0)
    return per_agent ? launch_blocks64<N, true, false, BF>(A, pb, s, nullptr)
                     : launch_blocks64<N, false, false, BF>(A, pb, s, nullptr);
  // small runs (the paper's IPPO setting is 16 envs per run): blocks of 32 or 16 envs inside a run
  if (A.E % 32 == 0)
    return per_agent ? rollout_impl<N, 32, 1, true, false, BF, 32>(A, pb, s) : rollout_impl<N, 32, 1, false, false, BF, 32>(A, pb, s);
  if (A.E % 16 == 0)
    return per_agent ? rollout_impl<N, 16, 1, true, false, BF, 32>(A, pb, s) : rollout_impl<N, 16, 1, false, false, BF, 32>(A, pb, s);
  *why = "with several runs, num_envs per run must be a multiple of 16";
  return hipSuccess;
  }
}

// Actor-critic rollout: 256 envs per block = four 64-env sync groups (12 wavefronts at N = 3)
// around one staged copy of the two networks (79 KB of the 160 KB LDS for fp32 weights) when that
// fills at least half of the CUs; 64-env blocks (one per CU) otherwise, and with several runs
// whose size is a multiple of 64 but not of 256.
template <int N, bool BF>
hipError_t launch_ac_n(const RolloutArgs& A, const PolicyBuffers& pb, const PolicyBuffers& critic, hipStream_t s,
                       const char** why) {
  const bool one_run = A.TE == A.E;
  const bool per_agent = A.ph.reward_mode == 1;
  if constexpr (N > 3) {
    // both staged images and the block's observation rows: 64 envs up to 6 agents, 32 envs with 7, 16 envs beyond
    static_assert(!BF, "bf16 weights with 4 and more agents are another kernel's");
    constexpr int kEnvs = N <= 6 ? 64 : (N == 7 ? 32 : 16);
    if (!one_run && A.E % kEnvs != 0) {
      *why = "with several runs and 4 or more agents, num_envs per run must be a multiple of 64 (of 32 with 7 agents, of 16 with 8 to 10)";
      return hipSuccess;
    }
    return per_agent ? rollout_impl<N, kEnvs, 1, true, true, false>(A, pb, s, critic.packed)
                     : rollout_impl<N, kEnvs, 1, false, true, false>(A, pb, s, critic.packed);
  } else {
  if (one_run ? A.TE / 256 >= compute_units() / 2 : A.E % 256 == 0)
    return per_agent ? rollout_impl<N, 256, 3, true, true, BF>(A, pb, s, critic.packed)
                     : rollout_impl<N, 256, 3, false, true, BF>(A, pb, s, critic.packed);
  if (one_run || A.E % 64 == 0)
    return per_agent ? launch_blocks64<N, true, true, BF>(A, pb, s, critic.packed)
                     : launch_blocks64<N, false, true, BF>(A, pb, s, critic.packed);
  if (A.E % 32 == 0)
    return per_agent ? rollout_impl<N, 32, 1, true, true, BF, 32>(A, pb, s, critic.packed)
                     : rollout_impl<N, 32, 1, false, true, BF, 32>(A, pb, s, critic.packed);
  if (A.E % 16 == 0)
    return per_agent ? rollout_impl<N, 16, 1, true, true, BF, 32>(A, pb, s, critic.packed)
                     : rollout_impl<N, 16, 1, false, true, BF, 32>(A, pb, s, critic.packed);
  *why = "with several runs, num_envs per run must be a multiple of 16";
  return hipSuccess;
  }
}

}  // namespace

// fp32 weights: 1..10 agents (the 4N + 2 live inputs of a row fill half a K slice of layer 1, one slice or
// two); bf16 weights: 1..3 (4 and more agents with bf16 weights run the lane-per-agent bf16 kernel)
bool f32_supported(int N, int H, bool bf16) { return H == kH && N >= 1 && N <= (bf16 ? 3 : 10); }

size_t packed_run_bytes_f32(int N, bool bf16) {
  if (bf16) return PkB::RUN_BYTES;
  const int kin = 4 * N + 2;
  return kin > 32 ? PkT<false, true, 2>::RUN_BYTES : (kin > 16 ? PkT<false, true>::RUN_BYTES : Pk::RUN_BYTES);
}

hipError_t pack_policy_f32(PolicyBuffers& pb, int N, int R, const float* W1, const float* b1, const float* W2,
                           const float* b2, const float* W3, const float* b3, int nout, bool bf16, hipStream_t s) {
  switch (N) {
    case 1: return pack_impl<1>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    case 2: return pack_impl<2>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    case 3: return pack_impl<3>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    case 4: return bf16 ? hipErrorInvalidValue : pack_impl<4>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 5: return bf16 ? hipErrorInvalidValue : pack_impl<5>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 6: return bf16 ? hipErrorInvalidValue : pack_impl<6>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 7: return bf16 ? hipErrorInvalidValue : pack_impl<7>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 8: return bf16 ? hipErrorInvalidValue : pack_impl<8>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 9: return bf16 ? hipErrorInvalidValue : pack_impl<9>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    case 10: return bf16 ? hipErrorInvalidValue : pack_impl<10>(pb, R, W1, b1, W2, b2, W3, b3, nout, false, s);
    default: return hipErrorInvalidValue;
  }
}

#define MPE_BY_N_AND_DTYPE(FN, ...)                                              \
  switch (N) {                                                                   \
    case 1: return bf16 ? FN<1, true>(__VA_ARGS__) : FN<1, false>(__VA_ARGS__);  \
    case 2: return bf16 ? FN<2, true>(__VA_ARGS__) : FN<2, false>(__VA_ARGS__);  \
    case 3: return bf16 ? FN<3, true>(__VA_ARGS__) : FN<3, false>(__VA_ARGS__);  \
    case 4: return bf16 ? hipErrorInvalidValue : FN<4, false>(__VA_ARGS__);      \
    case 5: return bf16 ? hipErrorInvalidValue : FN<5, false>(__VA_ARGS__);      \
    case 6: return bf16 ? hipErrorInvalidValue : FN<6, false>(__VA_ARGS__);      \
    case 7: return bf16 ? hipErrorInvalidValue : FN<7, false>(__VA_ARGS__);      \
    case 8: return bf16 ? hipErrorInvalidValue : FN<8, false>(__VA_ARGS__);      \
    case 9: return bf16 ? hipErrorInvalidValue : FN<9, false>(__VA_ARGS__);      \
    case 10: return bf16 ? hipErrorInvalidValue : FN<10, false>(__VA_ARGS__);    \
    default: return hipErrorInvalidValue;                                        \
  }

hipError_t launch_rollout_ac_f32(int N, bool bf16, const RolloutArgs& A, const PolicyBuffers& pb,
                                 const PolicyBuffers& critic, hipStream_t s, const char** why) {
  MPE_BY_N_AND_DTYPE(launch_ac_n, A, pb, critic, s, why)
}

hipError_t launch_rollout_policy_f32(int N, bool bf16, const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s,
                                     const char** why) {
  MPE_BY_N_AND_DTYPE(launch_n, A, pb, s, why)
}

}  // namespace mpe
