// Fused rollout: policy MLP forward (MFMA) -> Gumbel-max sampling (Philox) -> environment
// transition -> reward / auto-reset -> observation, T times inside one persistent kernel.
//
// Mapping.  A block owns EB consecutive environments; one lane owns one AGENT (row =
// env_local * N + agent), so a wavefront is 64 consecutive agent rows = four 16-row MFMA
// tiles.  The block keeps the current observations of its rows in an LDS tile that serves
// three readers: the coalesced 16-byte trajectory stores, the B operands of layer 1, and
// nothing else -- environment state itself stays in registers for all T steps.
//
// MLP on the matrix cores, transposed: H^T[hidden x rows] = W^T[hidden x in] * X^T[in x rows].
// With v_mfma_f32_16x16x4_f32 (and v_mfma_f32_16x16x32_bf16) the accumulator layout of one
// layer -- lane l holds column (row of the batch) l%16 and hidden units 16m + 4(l/16) + r --
// is exactly a B-operand layout for the next layer once the weights are stored with the
// matching K order, so activations never leave registers between layers.  Weights are
// packed once (mpe_set_policy) into that A-operand order and staged in LDS per block.
//
// This file holds the general kernel (bf16 operands, wide layers, many agents); the fp32
// headline shape has its own kernel in mpe_policy_f32.hip.
//
// Policy shape follows the paper's MPE setting (App. G, IPPO table: two tanh layers of width
// 64, parameters shared by all agents; Sec. 3.2 "PPO"); the scaled scenario uses width 128
// with bf16 operands and fp32 accumulation.
#include "mpe_policy_common.h"

namespace mpe {

namespace {

// LDS plan of one block (bytes).  The logits buffer and the new-position exchange share one
// region: within a phase each wavefront touches only its own 64 rows of it (logits first, then
// its agents' new positions), and block barriers separate that phase from the one in which
// every wavefront reads the positions.
template <int N, int H, bool BF16, int EB>
struct Smem {
  using S = Shape<N, H, BF16>;
  static constexpr int ROWS = EB * N;
  static constexpr bool kRewardInRegs = (N <= 4);   // every lane evaluates the N*N distances itself
  static constexpr size_t WEIGHTS = S::OFF_W3A;                   // W1A + W2A (W3A lives in registers)
  static constexpr size_t BIAS = S::BIAS_BYTES;
  static constexpr size_t OBS = size_t(ROWS) * S::D * 4 + 64;     // + zeroed tail for K padding reads
  static constexpr size_t ZP = size_t(ROWS) * 5 * 4;              // logits [row][5]; newpos [row] float2 inside
  static constexpr size_t DMIN = kRewardInRegs ? 0 : size_t(ROWS) * 4;
  static constexpr size_t OFF_BIAS = (WEIGHTS + 15) & ~size_t(15);
  static constexpr size_t OFF_OBS = OFF_BIAS + ((BIAS + 15) & ~size_t(15));
  static constexpr size_t OFF_ZP = OFF_OBS + ((OBS + 15) & ~size_t(15));
  static constexpr size_t OFF_DMIN = OFF_ZP + ((ZP + 15) & ~size_t(15));
  static constexpr size_t TOTAL = OFF_DMIN + ((DMIN + 15) & ~size_t(15));
};

// A-operand registers of layer 3 (5 outputs padded to one 16-wide tile), loaded once per kernel.
template <int N, int H, bool BF16>
struct W3Regs {
  using S = Shape<N, H, BF16>;
  f32x4 f[BF16 ? 1 : S::S2 / 4];
  bf16x8 b[BF16 ? S::S2 : 1];
  __device__ __forceinline__ void load(const uint8_t* __restrict__ run_weights, int lane) {
    if constexpr (BF16) {
#pragma unroll
      for (int s = 0; s < S::S2; ++s) b[s] = reinterpret_cast<const bf16x8*>(run_weights + S::OFF_W3A)[s * 64 + lane];
    } else {
#pragma unroll
      for (int s4 = 0; s4 < S::S2 / 4; ++s4) f[s4] = reinterpret_cast<const f32x4*>(run_weights + S::OFF_W3A)[s4 * 64 + lane];
    }
  }
};

// MLP forward of one 16-row tile (general kernel: bf16 operands, fp32 accumulation); rows'
// observations are in the LDS tile at obs_rows (row stride D floats).  wsm holds W1A then W2A,
// bias holds b1, b2, b3 (padded to 16).  Leaves logits of row j in zrows[j*5 .. j*5+4].
template <int N, int H, bool BF16>
__device__ __forceinline__ void policy_tile(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                            const W3Regs<N, H, BF16>& w3, const float* __restrict__ obs_rows,
                                            float* __restrict__ zrows, int lane) {
  static_assert(BF16, "the fp32 shape has its own pipelined kernel");
  using S = Shape<N, H, BF16>;
  constexpr int D = S::D, MT = S::MT;
  const int j = lane & 15, gq = lane >> 4;
  // Weights and biases are re-read from LDS for every tile on purpose: the addresses go through
  // an opaque zero offset, so the compiler cannot hoist ~100 registers of loop-invariant
  // operands out of the step loop (which would cost a wavefront of occupancy).  The offset is an
  // integer, not a laundered pointer, so the loads stay LDS (ds_read) instructions.
  {
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  f32x4 acc[MT];
  f32x4 hid[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = *reinterpret_cast<const f32x4*>(bias + 16 * m + 4 * gq);
  // ---- layer 1
  {
    const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + S::OFF_W1A);
#pragma unroll
    for (int s = 0; s < S::S1; ++s) {
      const float* src = obs_rows + j * D + 32 * s + 8 * gq;
      const f32x4 lo = *reinterpret_cast<const f32x4*>(src);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(src + 4);
      bf16x8 b;
#pragma unroll
      for (int e = 0; e < 4; ++e) { b[e] = __bf16(lo[e]); b[4 + e] = __bf16(hi[e]); }
#pragma unroll
      for (int m = 0; m < MT; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1[(m * S::S1 + s) * 64 + lane], b, acc[m], 0, 0, 0);
    }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
#pragma unroll
    for (int r = 0; r < 4; ++r) hid[m][r] = fast_tanh(acc[m][r]);
    acc[m] = *reinterpret_cast<const f32x4*>(bias + H + 16 * m + 4 * gq);
  }
  // ---- layer 2
  {
    const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + S::OFF_W2A);
#pragma unroll
    for (int s = 0; s < S::S2; ++s) {
      bf16x8 b;
#pragma unroll
      for (int e = 0; e < 4; ++e) { b[e] = __bf16(hid[2 * s][e]); b[4 + e] = __bf16(hid[2 * s + 1][e]); }
#pragma unroll
      for (int m = 0; m < MT; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w2[(m * S::S2 + s) * 64 + lane], b, acc[m], 0, 0, 0);
    }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
#pragma unroll
    for (int r = 0; r < 4; ++r) hid[m][r] = fast_tanh(acc[m][r]);
  }
  // ---- layer 3; two accumulators break the dependent chain
  f32x4 z0 = *reinterpret_cast<const f32x4*>(bias + 2 * H + 4 * gq);
  f32x4 z1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int s = 0; s < S::S2; ++s) {
    bf16x8 b;
#pragma unroll
    for (int e = 0; e < 4; ++e) { b[e] = __bf16(hid[2 * s][e]); b[4 + e] = __bf16(hid[2 * s + 1][e]); }
    if (s & 1) z1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.b[s], b, z1, 0, 0, 0);
    else z0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.b[s], b, z0, 0, 0, 0);
  }
  z0 += z1;
  // lane (j, gq) holds outputs 4gq + r of row j: outputs 0..3 in group 0, output 4 in group 1
  if (gq == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) zrows[j * 5 + r] = z0[r];
  } else if (gq == 1) {
    zrows[j * 5 + 4] = z0[0];
  }
}

// Cooperative copy of NF4 float4 from LDS to global by THREADS lanes; all reads issued first.
template <int NF4, int THREADS>
__device__ __forceinline__ void block_stream_out_full(const float* tile, float* dst, int tid) {
  constexpr int kFullIters = NF4 / THREADS;
  constexpr int kTail = NF4 % THREADS;
  const v4f* src4 = reinterpret_cast<const v4f*>(tile) + tid;
  v4f* dst4 = reinterpret_cast<v4f*>(dst) + tid;
  v4f v[kFullIters > 0 ? kFullIters : 1];
  v4f vt = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int k = 0; k < kFullIters; ++k) v[k] = src4[k * THREADS];
  if (kTail > 0 && tid < kTail) vt = src4[kFullIters * THREADS];
#pragma unroll
  for (int k = 0; k < kFullIters; ++k) dst4[k * THREADS] = v[k];
  if (kTail > 0 && tid < kTail) dst4[kFullIters * THREADS] = vt;
}

template <int N, int H, bool BF16, int EB, int MINW>
__global__ __launch_bounds__(EB * N, MINW) void rollout_policy_kernel(RolloutArgs A, const uint8_t* __restrict__ packed,
                                                                      int per_run_weights) {
  using S = Shape<N, H, BF16>;
  using M = Smem<N, H, BF16, EB>;
  constexpr int D = S::D, ROWS = EB * N, THREADS = ROWS;
  static_assert(THREADS % 64 == 0, "block must be whole wavefronts");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* wsm = smem;
  float* bias = reinterpret_cast<float*>(smem + M::OFF_BIAS);
  float* tile = reinterpret_cast<float*>(smem + M::OFF_OBS);
  float* zbuf = reinterpret_cast<float*>(smem + M::OFF_ZP);     // [ROWS][5]; wave w owns rows 64w..64w+63
  float* dminbuf = reinterpret_cast<float*>(smem + M::OFF_DMIN);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int el = tid / N, i = tid - el * N;          // env within block, agent
  const size_t TE = A.TE;
  const size_t g0 = size_t(blockIdx.x) * EB;
  const size_t g = g0 + el;
  const bool valid = g < TE;
  const uint32_t gc = valid ? uint32_t(g) : uint32_t(g0);
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;
  const size_t left = TE - g0;
  const int nvalid = left < size_t(EB) ? int(left) : EB;   // valid envs in this block
  // new-position slot of row r inside the shared logits/positions region: the first 8 bytes of
  // the 20-byte logits slot of that row's wavefront-local index
  auto newpos_of = [&](int r) -> float2* { return reinterpret_cast<float2*>(zbuf + (r >> 6) * (64 * 5)) + (r & 63); };

  // ---- stage this block's weights (the run of its first env): W1A, W2A, biases in LDS; W3A in registers
  const uint8_t* run_weights = packed + (per_run_weights ? size_t(uint32_t(g0) / A.E) * S::RUN_BYTES : 0);
  W3Regs<N, H, BF16> w3;
  w3.load(run_weights, lane);
  {
    const uint4* src = reinterpret_cast<const uint4*>(run_weights);
    uint4* dst = reinterpret_cast<uint4*>(wsm);
    for (int k = tid; k < int(S::OFF_W3A / 16); k += THREADS) dst[k] = src[k];
    const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + S::OFF_BIAS);
    uint4* bdst = reinterpret_cast<uint4*>(bias);
    for (int k = tid; k < int(S::BIAS_BYTES / 16); k += THREADS) bdst[k] = bsrc[k];
    if (tid < 16) tile[ROWS * D + tid] = 0.0f;
  }

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

  bool done_prev = false;
  const int n_out_floats = nvalid * N * D;  // floats of one time slice this block writes
  // Output addresses = uniform per-step base (advanced once per step, lives in SGPRs) + a
  // 32-bit lane offset that never changes.
  float* obs_p = A.obs_traj ? A.obs_traj + g0 * (N * D) : nullptr;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  const uint32_t row_off = uint32_t(gc) * N + i;      // index of this agent inside a time slice
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  uint32_t step = A.abs_step;

  for (int t = 0; t <= A.T; ++t, ++step) {
    __syncthreads();  // (A) tile (and dminbuf) complete
    if constexpr (!M::kRewardInRegs) {
      // reward and done of the step finished in the previous iteration
      if (t > 0) {
        if (env_writer) {
          if (rew_base) {
            float r = 0.0f;
#pragma unroll
            for (int a = 0; a < N; ++a) r -= dminbuf[el * N + a];
            (rew_base - TE)[gc] = r;
          }
          if (done_base) (done_base - TE)[gc] = done_prev ? 1 : 0;
        }
      }
    }
    // stream the tile out: obs_traj[t] for t < T, last_obs at t == T
    {
      float* dst = (t < A.T) ? obs_p : (A.last_obs ? A.last_obs + g0 * (N * D) : nullptr);
      if (dst) {
        const bool vec4 = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
        if (vec4 && nvalid == EB) {
          block_stream_out_full<ROWS * D / 4, THREADS>(tile, dst, tid);
        } else if (vec4) {
          const int n4 = n_out_floats >> 2;
          for (int k = tid; k < n4; k += THREADS)
            reinterpret_cast<float4*>(dst)[k] = reinterpret_cast<const float4*>(tile)[k];
          if ((n_out_floats & 2) && tid == 0)
            reinterpret_cast<float2*>(dst)[n_out_floats / 2 - 1] = reinterpret_cast<const float2*>(tile)[n_out_floats / 2 - 1];
        } else {
          for (int k = tid; k < (n_out_floats >> 1); k += THREADS)
            reinterpret_cast<float2*>(dst)[k] = reinterpret_cast<const float2*>(tile)[k];
        }
      }
      if (obs_p) obs_p += TE * (N * D);
    }
    if (t == A.T) break;

    // ---- policy: four 16-row tiles per wavefront
#pragma unroll 1
    for (int q = 0; q < 4; ++q) {
      const int r0 = wave * 64 + q * 16;
      policy_tile<N, H, BF16>(wsm, bias, w3, tile + r0 * D, zbuf + r0 * 5, lane);
    }
    wave_sync();
    float z[kNumActions];
#pragma unroll
    for (int k = 0; k < kNumActions; ++k) z[k] = zbuf[tid * 5 + k];
    const uint32_t act = gumbel_argmax(z, A.seed, run, env, step, uint32_t(i));
    if (act_base) {
      if (valid) act_base[row_off] = uint8_t(act);
      act_base += TE * N;
    }

    // ---- transition of this lane's agent
    float fx = A.ph.accel * action_dir_x(act);
    float fy = A.ph.accel * action_dir_y(act);
#pragma unroll
    for (int a = 0; a < N; ++a) {
      if (a != i) {
        const float dx = px - qx[a];
        const float dy = py - qy[a];
        const float k = contact_factor(dx, dy, A.ph);
        fx = fmaf(k, dx, fx);
        fy = fmaf(k, dy, fy);
      }
    }
    px = fmaf(vx, A.ph.dt, px);
    py = fmaf(vy, A.ph.dt, py);
    vx = fmaf(fx, A.ph.dt_over_mass, vx * A.ph.keep);
    vy = fmaf(fy, A.ph.dt_over_mass, vy * A.ph.keep);
    wave_sync();      // every lane of this wavefront has read its logits: the slots may be reused
    *newpos_of(tid) = make_float2(px, py);
    __syncthreads();  // (C) new positions visible; everyone is done reading the tile

#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float2 p = *newpos_of(el * N + a);
      qx[a] = p.x;
      qy[a] = p.y;
    }
    if constexpr (M::kRewardInRegs) {
      // shared coverage reward, evaluated by every lane (N*N distances), stored by agent 0
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
      if (rew_base && env_writer) rew_base[gc] = r;
    } else {
      // coverage term of landmark i: min over agents of the distance to it
      float mylx = 0.0f, myly = 0.0f;
#pragma unroll
      for (int l = 0; l < N; ++l) {
        if (l == i) { mylx = lx[l]; myly = ly[l]; }
      }
      float best2 = INFINITY;
#pragma unroll
      for (int a = 0; a < N; ++a) {
        const float dx = qx[a] - mylx, dy = qy[a] - myly;
        best2 = fminf(best2, fmaf(dx, dx, dy * dy));
      }
      dminbuf[tid] = hw_sqrt(best2);
    }
    ep += 1;
    done_prev = ep >= A.ph.max_ep;
    if constexpr (M::kRewardInRegs) {
      if (done_base && env_writer) done_base[gc] = done_prev ? 1 : 0;
    }
    if (rew_base) rew_base += TE;
    if (done_base) done_base += TE;
    if (done_prev) {
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

template <int N, int H, bool BF16>
hipError_t pack_impl(PolicyBuffers& pb, int R, const float* W1, const float* b1, const float* W2,
                     const float* b2, const float* W3, const float* b3, hipStream_t s) {
  using S = Shape<N, H, BF16>;
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * S::RUN_BYTES); e != hipSuccess) return e;
  const int total = int(S::RUN_BYTES / S::ELT);  // upper bound on elements of one run
  dim3 grid(cdiv(total, 256), R);
  hipLaunchKernelGGL((pack_policy_kernel<N, H, BF16>), grid, dim3(256), 0, s,
                     static_cast<uint8_t*>(pb.packed), W1, b1, W2, b2, W3, b3);
  return hipGetLastError();
}

template <int N, int H, bool BF16, int EB, int MINW>
hipError_t rollout_impl(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s) {
  using M = Smem<N, H, BF16, EB>;
  const dim3 grid((A.TE + EB - 1) / EB);
  auto kern = rollout_policy_kernel<N, H, BF16, EB, MINW>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(M::TOTAL));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(EB * N), M::TOTAL, s, A, static_cast<const uint8_t*>(pb.packed),
                     int(A.TE != A.E));
  return hipGetLastError();
}

}  // namespace

// General shapes built: (N, H, envs per block, min waves per SIMD), bf16 operands.
#define MPE_WIDE_CASES(X) X(10, 128, 32, 2)

bool wide_supported(int N, int H) {
#define X(N_, H_, EB_, MW_) if (N == N_ && H == H_) return true;
  MPE_WIDE_CASES(X)
#undef X
  return false;
}

hipError_t pack_policy_wide(PolicyBuffers& pb, int N, int H, int R, const float* W1, const float* b1,
                            const float* W2, const float* b2, const float* W3, const float* b3, hipStream_t s) {
#define X(N_, H_, EB_, MW_) if (N == N_ && H == H_) return pack_impl<N_, H_, true>(pb, R, W1, b1, W2, b2, W3, b3, s);
  MPE_WIDE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

hipError_t launch_rollout_policy_wide(int N, int H, const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s,
                                      const char** why) {
#define X(N_, H_, EB_, MW_)                                                                      \
  if (N == N_ && H == H_) {                                                                      \
    if (A.TE != A.E && (A.E % EB_) != 0) {                                                       \
      *why = "with several runs, num_envs per run must be a multiple of the block's env count";  \
      return hipSuccess;                                                                         \
    }                                                                                            \
    return rollout_impl<N_, H_, true, EB_, MW_>(A, pb, s);                                       \
  }
  MPE_WIDE_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace mpe
