// Fused rollout for wide shapes: many agents, wide hidden layers, bf16 operands with fp32
// accumulation (the scaled scenario: 10 agents, 60 -> 128 -> 128 -> 5).  Policy MLP forward
// (MFMA) -> Gumbel-max sampling (Philox) -> environment transition -> reward / auto-reset ->
// observation, T times inside one persistent kernel.  The fp32 headline shape has its own kernel
// in mpe_policy_f32.hip.
//
// Policy shape follows the paper's MPE setting (App. G, IPPO table: two tanh layers, parameters
// shared by all agents; Sec. 3.2 "PPO"), widened to 128 with bf16 operands.
//
// Mapping.  A block owns EB consecutive environments; one lane owns one AGENT (row =
// env_local * N + agent), so a wavefront is 64 consecutive agent rows = four 16-row MFMA tiles.
// Environment state and the lane's own observation row stay in registers for all T steps.
//
// Keeping LDS small is what buys occupancy here (the packed weights alone are 49 KB per block),
// so the observation rows never sit in LDS as a whole:
//  * B operands of layer 1: the lane rounds its row to bf16 in registers; the matrix instruction
//    wants lane (j, g) to hold 8 consecutive inputs (chunk g) of row 16c + j for tile c, and the
//    owner of that row is lane (j, c): a 4 x 4 transpose between register index and lane group,
//    done with v_permlane32_swap + v_permlane16_swap, no memory involved.
//  * trajectory stores: every lane stores its own row straight from registers as 16-byte
//    chunks.  (Measured alternatives: staging 16 rows at a time through LDS makes the stores
//    contiguous but costs 60 quarter-occupied ds_write_b128 per wavefront and step -- an LDS
//    write costs ~13.5 cycles per CU whatever its lane count -- and came out slower.)
//  * layers 2 and 3: the accumulator layout of one layer -- lane (j, g) holds batch row j and
//    hidden units 16m + 4g + r -- is a B-operand layout for the next layer once the weights are
//    packed in the matching K order, so activations never leave registers.
// The only data that cross wavefronts are the new positions and the per-landmark coverage
// distances of an env's agents (double-buffered by step parity): one barrier per step.
//
// Occupancy.  At ~168 registers a SIMD holds three wavefronts, and the hardware places a block's
// wavefronts on the four SIMDs as a unit: two 5-wavefront blocks do not fit one CU (measured:
// one resident block per CU), a 10-wavefront block does (3 + 3 + 2 + 2).  So a block is TWO
// independent 32-env groups that share the staged weights, and the per-step barrier is per group:
// an arrival counter in LDS instead of the block barrier, so that a group never waits for the other.
//
// Balance (10 agents).  640 rows are ten wavefronts of 64, which the four SIMDs can only hold as
// 3 + 3 + 2 + 2: two SIMDs idle a third of the time (measured: vector and matrix units together busy
// 83 % of the SIMD cycles).  The network is work per 16-row TILE, 40 tiles per block, so the 10-agent
// shape runs TWELVE wavefronts instead, three per SIMD, that own 4, 3 and 3 tiles (64, 48, 48 rows;
// the last 16 lanes of a 48-row wavefront own no row and store nothing): ten tiles on every SIMD.
#include "mpe_policy_common.h"

namespace mpe {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Packed weight layout of one run (bf16): A operands of v_mfma_f32_16x16x32_bf16, lane (i = lane%16,
// gq = lane/16) holds weights [k = 8 gq + e][out = 16 m + i], e = 0..7 (16 bytes).
//   W1A [m][s][lane]  layer 1, K slices of 32 inputs in natural order, zero padded past the
//                     4N + 2 live observation entries
//   W2A [m][s][lane]  layer 2, K position (s, gq, e) = hidden unit hidden_of(s, gq, e): the order
//                     in which the accumulators of the previous layer hold the hidden units
//   W3A [s][lane]     layer 3 (5 outputs padded to 16)
//   bias b1 [H], b2 [H], b3 [16] fp32
template <int N, int H>
struct Shape {
  static constexpr int D = 6 * N;
  static constexpr int KIN = 4 * N + 2;           // non-zero leading entries of an observation
  static constexpr int KS = 32;                   // K extent of one MFMA
  static constexpr int MT = H / 16;               // 16-wide tiles of hidden units
  static constexpr int S1 = cdiv(KIN, KS);        // K slices of layer 1
  static constexpr int S2 = H / KS;               // K slices of layers 2 and 3
  static constexpr size_t W1A_BYTES = size_t(MT) * S1 * 64 * 16;
  static constexpr size_t W2A_BYTES = size_t(MT) * S2 * 64 * 16;
  static constexpr size_t W3A_BYTES = size_t(S2) * 64 * 16;
  static constexpr size_t BIAS_BYTES = size_t(2 * H + 16) * 4;
  static constexpr size_t OFF_W1A = 0;
  static constexpr size_t OFF_W2A = OFF_W1A + W1A_BYTES;
  static constexpr size_t OFF_W3A = OFF_W2A + W2A_BYTES;
  static constexpr size_t OFF_BIAS = OFF_W3A + W3A_BYTES;
  static constexpr size_t RUN_BYTES = OFF_BIAS + BIAS_BYTES;
};

// Hidden unit that K position (slice s, lane group gq, element e) of layers 2/3 refers to:
// the accumulator register (tile m, r) of lane group gq holds unit 16m + 4gq + r.
__host__ __device__ constexpr int hidden_of(int s, int gq, int e) { return 32 * s + 16 * (e / 4) + 4 * gq + (e % 4); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// One thread per packed element of one run (weights rounded to bf16, ties to even).
// nout = outputs of the network: 5 (policy) or 1 (critic; W3 [H], b3 [1] per run).
template <int N, int H>
__global__ void pack_policy_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                   const float* __restrict__ b1, const float* __restrict__ W2,
                                   const float* __restrict__ b2, const float* __restrict__ W3,
                                   const float* __restrict__ b3, int nout) {
  using S = Shape<N, H>;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * S::RUN_BYTES;
  W1 += size_t(run) * S::D * H;
  b1 += size_t(run) * H;
  W2 += size_t(run) * H * H;
  b2 += size_t(run) * H;
  W3 += size_t(run) * H * nout;
  b3 += size_t(run) * nout;
  constexpr int n1 = S::MT * S::S1 * 64 * 8, n2 = S::MT * S::S2 * 64 * 8, n3 = S::S2 * 64 * 8, nb = 2 * H + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  auto put = [&](size_t off, int i, float v) { reinterpret_cast<uint16_t*>(out + off)[i] = f32_to_bf16_rne(v); };
  if (idx < n1) {   // [m][s][lane][e]; k = 32 s + 8 gq + e (natural order)
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % S::S1, m = idx / (512 * S::S1);
    const int k = S::KS * s + 8 * (lane / 16) + e, o = 16 * m + lane % 16;
    put(S::OFF_W1A, idx, k < S::KIN ? W1[size_t(k) * H + o] : 0.0f);
    return;
  }
  idx -= n1;
  if (idx < n2) {   // [m][s][lane][e]
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % S::S2, m = idx / (512 * S::S2);
    put(S::OFF_W2A, idx, W2[size_t(hidden_of(s, lane / 16, e)) * H + 16 * m + lane % 16]);
    return;
  }
  idx -= n2;
  if (idx < n3) {   // [s][lane][e]
    const int e = idx % 8, lane = (idx / 8) % 64, s = idx / 512, o = lane % 16;
    put(S::OFF_W3A, idx, o < nout ? W3[size_t(hidden_of(s, lane / 16, e)) * nout + o] : 0.0f);
    return;
  }
  idx -= n3;
  if (idx < nb) {
    float v;
    if (idx < H) v = b1[idx];
    else if (idx < 2 * H) v = b2[idx - H];
    else v = (idx - 2 * H) < nout ? b3[idx - 2 * H] : 0.0f;
    reinterpret_cast<float*>(out + S::OFF_BIAS)[idx] = v;
  }
}

// LDS plan of one block (bytes).
// UNIFORM (no policy: seeded uniform actions): no weights; the stage holds one 16-row tile of
// observations on its way to the trajectory.
// AC (actor-critic rollout): the critic's packed image follows the policy's, and every wavefront has a
// second stage for the critic's outputs.
// Envs of one sync group: the smallest count whose agent rows fill whole wavefronts.
__host__ __device__ constexpr int sync_group_envs(int n) {
  int g = 64;
  while (g > 1 && (n % 2 == 0)) { g /= 2; n /= 2; }
  return g;
}

// Rows -> wavefronts.  Plain: wavefront w owns rows 64 w .. 64 w + 63.  Balanced (10 agents, two 32-env
// sync groups of 320 rows = 20 tiles): six wavefronts per group own 4, 4, 3, 3, 3, 3 tiles; the hardware
// deals wavefront h of a block to SIMD h % 4 and group g gets the hardware wavefronts g, g + 2, g + 4, ...,
// so wavefronts 0, 2, 4 of a group share one SIMD and 1, 3, 5 another: 4 + 3 + 3 tiles each.
template <int N, int EB, bool UNIFORM>
struct RowMap {
  static constexpr bool kBalanced = (N == 10 && EB == 64 && !UNIFORM);
  static constexpr int ROWS = EB * N;
  static constexpr int GE = sync_group_envs(N);                     // envs of one sync group
  static constexpr int GW = kBalanced ? 6 : GE * N / 64;            // wavefronts of one sync group
  static constexpr int WAVES = kBalanced ? 12 : ROWS / 64;
  // first row and row count of wavefront v of a group (row numbers inside the group)
  __host__ __device__ static constexpr int first_row(int v) { return kBalanced ? (v < 2 ? 64 * v : 128 + 48 * (v - 2)) : 64 * v; }
  __host__ __device__ static constexpr int rows_of(int v) { return kBalanced ? (v < 2 ? 64 : 48) : 64; }
};

template <int N, int H, int EB, bool UNIFORM = false, bool AC = false>
struct Smem {
  using S = Shape<N, H>;
  static constexpr int ROWS = EB * N, WAVES = RowMap<N, EB, UNIFORM>::WAVES;
  static constexpr size_t WEIGHTS = UNIFORM ? 0 : S::OFF_BIAS;     // W1A + W2A + W3A
  static constexpr size_t OFF_BIAS = WEIGHTS;
  static constexpr size_t OFF_CRITIC = OFF_BIAS + (UNIFORM ? 0 : S::BIAS_BYTES);   // AC: W1A, W2A, W3A, biases of the critic
  static constexpr size_t STAGE_WAVE = UNIFORM ? size_t(16) * S::D * 4 : size_t(64) * 5 * 4;   // else the wave's logits [64][5] (AC: first the values)
  static constexpr size_t OFF_STAGE = OFF_CRITIC + (AC ? S::RUN_BYTES : 0);
  static constexpr size_t OFF_NEWPOS = OFF_STAGE + WAVES * STAGE_WAVE;   // [2][ROWS] float2, by step parity
  static constexpr size_t OFF_DMIN = OFF_NEWPOS + size_t(2) * ROWS * 8;  // [2][ROWS] float,  by step parity
  static constexpr size_t OFF_LM = OFF_DMIN + size_t(2) * ROWS * 4;      // [EB][N] float2 landmark positions
  static constexpr size_t OFF_RESPOS = OFF_LM + size_t(ROWS) * 8;        // [EB][N] float2 positions after a reset
  static constexpr size_t OFF_ARRIVED = OFF_RESPOS + size_t(ROWS) * 8;   // arrival counter of each sync group
  static constexpr size_t TOTAL = OFF_ARRIVED + 16;
  static_assert(OFF_STAGE % 16 == 0 && STAGE_WAVE % 16 == 0 && OFF_NEWPOS % 16 == 0 && OFF_CRITIC % 16 == 0, "alignment");
  static_assert(TOTAL <= 160 * 1024 && !(UNIFORM && AC), "LDS");
};

// Round two floats to bf16 (nearest even) and pack them: low half <- a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// tanh of 8 accumulator values (hidden tiles 2s and 2s+1 of one batch tile), rounded to bf16: the
// B operand of K slice s of the next layer (element e <-> tile 2s + e/4, register e%4).
__device__ __forceinline__ bf16x8 tanh_pack(const f32x4& a0, const f32x4& a1) {
  u32x4 p;
  p[0] = pack_bf16(fast_tanh(a0[0]), fast_tanh(a0[1]));
  p[1] = pack_bf16(fast_tanh(a0[2]), fast_tanh(a0[3]));
  p[2] = pack_bf16(fast_tanh(a1[0]), fast_tanh(a1[1]));
  p[3] = pack_bf16(fast_tanh(a1[2]), fast_tanh(a1[3]));
  return __builtin_bit_cast(bf16x8, p);
}

#define MPE_MFMA_BF(A, B, C) __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, C, 0, 0, 0)

// MLP forward of one 16-row tile from its layer-1 B operands b1[slice].  wsm holds W1A then W2A,
// then W3A, bias holds b1, b2, b3 (padded to 16).  Leaves the logits of row j in
// zrows[j*5 .. j*5+4].
template <int N, int H>
__device__ __forceinline__ void policy_tile(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                            const bf16x8 (&b1)[Shape<N, H>::S1], float* __restrict__ zrows,
                                            int lane) {
  using S = Shape<N, H>;
  constexpr int MT = S::MT;
  const int j = lane & 15, gq = lane >> 4;
  __builtin_amdgcn_s_setprio(2);   // the network goes ahead of the vector-only env step of other wavefronts
  // Weights and biases are re-read from LDS for every tile on purpose: the addresses go through
  // an opaque zero offset, so the compiler cannot hoist loop-invariant operands out of the step
  // loop (which would cost registers and a wavefront of occupancy).  The offset is an integer,
  // not a laundered pointer, so the loads stay LDS (ds_read) instructions.
  {
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + S::OFF_W1A) + lane;   // [m][s][lane]
  const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + S::OFF_W2A) + lane;   // [m][s][lane]
  const bf16x8* w3 = reinterpret_cast<const bf16x8*>(wsm + S::OFF_W3A) + lane;   // [s][lane]
  // The A operands of layers 1 and 2 are used in the order k = (layer, slice, m); a ring of kAhead
  // of them is kept in flight so that an LDS read is issued kAhead matrix instructions before
  // the one that consumes it.
  constexpr int K1 = S::S1 * MT, K2 = S::S2 * MT, kAhead = 4;
  auto a_ptr = [&](int k) -> const bf16x8* {
    return k < K1 ? w1 + ((k % MT) * S::S1 + k / MT) * 64 : w2 + (((k - K1) % MT) * S::S2 + (k - K1) / MT) * 64;
  };
  bf16x8 ring[kAhead];
#pragma unroll
  for (int k = 0; k < kAhead; ++k) ring[k] = *a_ptr(k);
  f32x4 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = *reinterpret_cast<const f32x4*>(bias + 16 * m + 4 * gq);
#pragma unroll
  for (int k = 0; k < K1; ++k) {
    acc[k % MT] = MPE_MFMA_BF(ring[k % kAhead], b1[k / MT], acc[k % MT]);
    ring[k % kAhead] = *a_ptr(k + kAhead);
  }
  bf16x8 hb[S::S2];
#pragma unroll
  for (int s = 0; s < S::S2; ++s) hb[s] = tanh_pack(acc[2 * s], acc[2 * s + 1]);
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = *reinterpret_cast<const f32x4*>(bias + H + 16 * m + 4 * gq);
#pragma unroll
  for (int k = K1; k < K1 + K2; ++k) {
    acc[k % MT] = MPE_MFMA_BF(ring[k % kAhead], hb[(k - K1) / MT], acc[k % MT]);
    if (k + kAhead < K1 + K2) ring[k % kAhead] = *a_ptr(k + kAhead);
  }
  // layer 3; two accumulators break the dependent chain
  f32x4 z0 = *reinterpret_cast<const f32x4*>(bias + 2 * H + 4 * gq);
  f32x4 z1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int s = 0; s < S::S2; ++s) {
    const bf16x8 b = tanh_pack(acc[2 * s], acc[2 * s + 1]);
    if (s & 1) z1 = MPE_MFMA_BF(w3[s * 64], b, z1);
    else z0 = MPE_MFMA_BF(w3[s * 64], b, z0);
  }
  z0 += z1;
  __builtin_amdgcn_s_setprio(0);
  // lane (j, gq) holds outputs 4gq + r of row j: outputs 0..3 in group 0, output 4 in group 1
  if (gq == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) zrows[j * 5 + r] = z0[r];
  } else if (gq == 1) {
    zrows[j * 5 + 4] = z0[0];
  }
}

// PER_AGENT: rew_traj is [T][TE][N], the mixed per-agent reward; every lane stores its agent's.
// UNIFORM: no policy; every agent's action is the seeded uniform draw.  The kernel is then bound
// by the trajectory stores, and the observation rows leave 16 at a time through the wave's LDS
// stage as contiguous 3,840-byte pieces (per-lane stores of 240-byte rows sustain only ~3 TB/s).
// AC: a critic of the same shape with one output (`packed_critic`) is evaluated on every observation
// acted on; its value and the log-probability of the sampled action are recorded (paper Sec. 3.2: IPPO).
template <int N, int H, int EB, int MINW, bool PER_AGENT, bool UNIFORM, bool AC = false>
__global__ __launch_bounds__((RowMap<N, EB, UNIFORM>::WAVES * 64), MINW) void rollout_policy_kernel(RolloutArgs A, const uint8_t* __restrict__ packed,
                                                                      const uint8_t* __restrict__ packed_critic,
                                                                      int per_run_weights, uint32_t groups,
                                                                      uint32_t groups_per_xcd) {
  using S = Shape<N, H>;
  using M = Smem<N, H, EB, UNIFORM, AC>;
  using RM = RowMap<N, EB, UNIFORM>;
  constexpr int D = S::D, KIN = S::KIN, ROWS = EB * N, THREADS = RM::WAVES * 64;
  constexpr int RF4 = D / 4;                 // 16-byte chunks of one observation row
  constexpr int PD = S::S1 * 16;             // dwords of one row as bf16 pairs, zero padded to whole K slices
  constexpr int GE = RM::GE, GW = RM::GW;                    // envs / wavefronts of one sync group
  static_assert(EB % GE == 0 && EB / GE <= 4, "a block is whole sync groups");
  static_assert(D % 2 == 0 && KIN % 2 == 0,
                "rows are stored as 16-byte chunks (8-byte with an odd agent count) and packed as bf16 pairs");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* wsm = smem;
  float* bias = reinterpret_cast<float*>(smem + M::OFF_BIAS);
  float2* newpos = reinterpret_cast<float2*>(smem + M::OFF_NEWPOS);
  float* dminbuf = reinterpret_cast<float*>(smem + M::OFF_DMIN);
  float2* lmbuf = reinterpret_cast<float2*>(smem + M::OFF_LM);
  float2* respos = reinterpret_cast<float2*>(smem + M::OFF_RESPOS);

  // Wavefront -> rows: the GW wavefronts of sync group g are the hardware wavefronts g, g + G, g + 2G, ...
  // (G groups per block).  The hardware deals a block's wavefronts to the four SIMDs in turn, so a
  // group then lives on 4 / G of the SIMDs and a wavefront waiting at the group's barrier yields its
  // issue slots to wavefronts of its own group.  `wave` and `tid` are these virtual indices: row = tid.
  const int lane = threadIdx.x & 63;
  const int hw_wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
  constexpr int kGroups = EB / GE;
  const int wave = kGroups > 1 ? (hw_wave % kGroups) * GW + hw_wave / kGroups : hw_wave;
  const int wv = wave % GW;                          // wavefront inside its sync group
  const int wave_first = (wave / GW) * (GE * N) + RM::first_row(wv);   // its first row inside the block
  const int wave_count = RM::rows_of(wv);            // rows it owns: 64, or 48 (three tiles) in the balanced map
  const bool active = !RM::kBalanced || lane < wave_count;   // false for the 16 spare lanes of a 48-row wavefront:
  const int tid = wave_first + (active ? lane : 0);           // they shadow the wavefront's first row and store nothing
  const int el = tid / N, i = tid - el * N;          // env within block, agent
  float* stage = reinterpret_cast<float*>(smem + M::OFF_STAGE + size_t(wave) * M::STAGE_WAVE);
  uint32_t* arrived = reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED) + wave / GW;
  const size_t TE = A.TE;
  // XCD-aware mapping: the hardware deals block b to XCD b % 8; each XCD gets one contiguous range
  // of env groups, so the partial cache lines of neighbouring groups meet in one L2.
  const uint32_t grp = (blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3);
  if (grp >= groups) return;  // whole block, before any barrier
  const size_t g0 = size_t(grp) * EB;
  const size_t g = g0 + el;
  const bool valid = active && g < TE;
  const uint32_t gc = valid ? uint32_t(g) : uint32_t(g0);
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;
  const size_t left = TE - g0;
  const int nvalid = left < size_t(EB) ? int(left) : EB;   // valid envs in this block
  const int wave_rows = min(max(nvalid * N - wave_first, 0), wave_count);   // rows of this wavefront that belong to valid envs

  // ---- stage this block's weights (the run of its first env) in LDS: the packed buffer is
  // W1A, W2A, W3A, biases in that order, and so is the LDS image
  if constexpr (!UNIFORM) {
    const uint8_t* run_weights = packed + (per_run_weights ? size_t(uint32_t(g0) / A.E) * S::RUN_BYTES : 0);
    const uint4* src = reinterpret_cast<const uint4*>(run_weights);
    uint4* dst = reinterpret_cast<uint4*>(wsm);
    for (int k = threadIdx.x; k < int(S::RUN_BYTES / 16); k += THREADS) dst[k] = src[k];
    if constexpr (AC) {
      const uint4* csrc = reinterpret_cast<const uint4*>(
          packed_critic + (per_run_weights ? size_t(uint32_t(g0) / A.E) * S::RUN_BYTES : 0));
      uint4* cdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC);
      for (int k = threadIdx.x; k < int(S::RUN_BYTES / 16); k += THREADS) cdst[k] = csrc[k];
    }
  }

  // ---- registers: own agent and landmark i (the one whose coverage distance this lane
  // evaluates).  LDS: all landmarks of the block's envs (they change only at a reset) and the
  // positions of all agents: the other agents' positions are read where they are needed
  // (observation, contacts, reward) instead of being held in 2N registers through the policy.
  // `cur` is where the env's current positions are: the exchange buffer of the latest step, or
  // `respos` when the env has just been reset (or at the start of the call).
  float px = 0.0f, py = 0.0f, vx = 0.0f, vy = 0.0f, mylx = 0.0f, myly = 0.0f;
  int32_t ep = 0;
  if (g < TE) {   // (a spare lane loads the row it shadows)
    px = A.st.pos_a[(0 * N + i) * TE + g];
    py = A.st.pos_a[(1 * N + i) * TE + g];
    mylx = A.st.pos_l[(0 * N + i) * TE + g];
    myly = A.st.pos_l[(1 * N + i) * TE + g];
    vx = A.st.vel_a[(0 * N + i) * TE + g];
    vy = A.st.vel_a[(1 * N + i) * TE + g];
    ep = A.st.ep_step[g];
  }
  if (active) {
    respos[tid] = make_float2(px, py);
    lmbuf[tid] = make_float2(mylx, myly);   // tid = el * N + i
  }
  const float2* cur = respos + el * N;
  if (threadIdx.x < EB / GE) reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED)[threadIdx.x] = 0u;
  __syncthreads();  // weights, biases, landmarks and counters staged; the only block-wide barrier

  // The lane's observation: its KIN leading entries (the trailing communication slots are zeros).
  auto build_obs = [&](float (&o)[KIN]) {
    o[0] = vx; o[1] = vy; o[2] = px; o[3] = py;
#pragma unroll
    for (int l = 0; l < N; ++l) {
      const float2 lm = lmbuf[el * N + l];
      o[4 + 2 * l] = lm.x - px;
      o[5 + 2 * l] = lm.y - py;
    }
    float2 q[N];
#pragma unroll
    for (int a = 0; a < N; ++a) q[a] = cur[a];
#pragma unroll
    for (int c = 0; c < N - 1; ++c) {   // other agents, ascending: slot c holds agent c + (c >= i)
      const float ox = c >= i ? q[c + 1].x : q[c].x;
      const float oy = c >= i ? q[c + 1].y : q[c].y;
      o[4 + 2 * N + 2 * c] = ox - px;
      o[5 + 2 * N + 2 * c] = oy - py;
    }
  };
  // Store this wavefront's rows to dst (its slot in a [env][N][D] slice).
  auto flush_rows = [&](const float (&o)[KIN], float* dst) {
    if constexpr (UNIFORM) {
      // rows of 6N floats: whole 16-byte chunks when N is even, 8-byte ones when it is odd
      constexpr int CW = D % 4 == 0 ? 4 : 2, RFC = D / CW;
      typedef float vC __attribute__((ext_vector_type(CW)));
      vC* stc = reinterpret_cast<vC*>(stage);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        wave_sync();  // the stage is free (previous readers done)
        if ((lane >> 4) == c) {
#pragma unroll
          for (int q = 0; q < RFC; ++q) {
            vC v;
#pragma unroll
            for (int e = 0; e < CW; ++e) v[e] = (CW * q + e < KIN) ? o[(CW * q + e < KIN) ? CW * q + e : 0] : 0.0f;
            stc[(lane & 15) * RFC + q] = v;
          }
        }
        wave_sync();
        const int nc = min(max(wave_rows - 16 * c, 0), 16) * RFC;   // chunks of this tile that are valid
        constexpr int kRounds = (16 * RFC + 63) / 64;
        vC v[kRounds];
#pragma unroll
        for (int rd = 0; rd < kRounds; ++rd)
          if (rd * 64 + lane < nc) v[rd] = stc[rd * 64 + lane];
        vC* dc = reinterpret_cast<vC*>(dst) + c * (16 * RFC);
#pragma unroll
        for (int rd = 0; rd < kRounds; ++rd)
          if (rd * 64 + lane < nc) __builtin_nontemporal_store(v[rd], &dc[rd * 64 + lane]);
      }
      wave_sync();
    } else if (lane < wave_rows) {
      if constexpr (D % 4 == 0) {
        v4f* d4 = reinterpret_cast<v4f*>(dst) + lane * RF4;
#pragma unroll
        for (int q = 0; q < RF4; ++q) {
          v4f v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (4 * q + e < KIN) ? o[(4 * q + e < KIN) ? 4 * q + e : 0] : 0.0f;
          d4[q] = v;
        }
      } else {   // odd agent counts: rows of 24 N bytes are only 8-byte aligned
        v2f* d2 = reinterpret_cast<v2f*>(dst) + lane * (D / 2);
#pragma unroll
        for (int q = 0; q < D / 2; ++q) {
          v2f v;
          v[0] = (2 * q < KIN) ? o[(2 * q < KIN) ? 2 * q : 0] : 0.0f;
          v[1] = (2 * q < KIN) ? o[(2 * q < KIN) ? 2 * q + 1 : 0] : 0.0f;
          d2[q] = v;
        }
      }
    }
  };

  // The lane's observation as bf16 pairs -> the layer-1 B operands of the wave's four 16-row tiles.
  [[maybe_unused]] auto pack_operands = [&](const float (&o)[KIN], bf16x8 (&b1)[4][S::S1]) {
    uint32_t pk[PD];
#pragma unroll
    for (int d = 0; d < PD; ++d) pk[d] = (2 * d < KIN) ? pack_bf16(o[(2 * d < KIN) ? 2 * d : 0], o[(2 * d < KIN) ? 2 * d + 1 : 0]) : 0u;
    // chunk g of slice s = dwords 16 s + 4 g .. + 3 of the packed row
#pragma unroll
    for (int s = 0; s < S::S1; ++s) {
      u32x4 tile_b[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t v[4] = {pk[16 * s + d], pk[16 * s + 4 + d], pk[16 * s + 8 + d], pk[16 * s + 12 + d]};
        transpose_groups(v);
#pragma unroll
        for (int c = 0; c < 4; ++c) tile_b[c][d] = v[c];
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) b1[c][s] = __builtin_bit_cast(bf16x8, tile_b[c]);
    }
  };
  [[maybe_unused]] const uint8_t* csm = smem + M::OFF_CRITIC;                                        // AC only
  [[maybe_unused]] const float* cbias = reinterpret_cast<const float*>(smem + M::OFF_CRITIC + S::OFF_BIAS);
  [[maybe_unused]] float* logp_base = A.logp_traj;
  [[maybe_unused]] float* value_base = A.value_traj;

  const size_t wave_row0 = (g0 * N + size_t(wave_first)) * D;  // float offset of this wavefront's rows in a slice
  float* obs_p = A.obs_traj ? A.obs_traj + wave_row0 : nullptr;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  const size_t row_off = size_t(gc) * N + i;          // index of this agent inside a time slice (can pass 2^32)
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  uint32_t step = A.abs_step;
  uint32_t overlaps = 0;   // PER_AGENT: other agents this one overlapped after the latest step

  // Reward of the step whose coverage distances are in dminbuf[parity]: their sum (negated) per env,
  // or, PER_AGENT, mixed with the lane's overlap count of that step.  Advances rew_base.
  auto store_reward = [&](int parity) {
    if (!rew_base) return;
    if (PER_AGENT ? valid : env_writer) {
      const float* dm = dminbuf + parity * ROWS + el * N;
      float r = 0.0f;
#pragma unroll
      for (int a = 0; a < N; ++a) r -= dm[a];
      if constexpr (PER_AGENT) rew_base[row_off] = mixed_reward(r, overlaps, A.ph);
      else rew_base[gc] = r;
    }
    rew_base += PER_AGENT ? TE * N : TE;
  };

  for (int t = 0; t < A.T; ++t, ++step) {
    // ---- observation row -> trajectory, and -> bf16 B operands of layer 1 for the wave's 4 tiles
    bf16x8 b1[4][S::S1];
    uint32_t act;
    if constexpr (UNIFORM) {
      if (obs_p) {
        float o[KIN];
        build_obs(o);
        flush_rows(o, obs_p);
        obs_p += TE * (N * D);
      }
      act = word_to_action(philox4x32_10(env, step, uint32_t(i), kTagUniformAction, A.seed, run).x);
    } else {
      float o[KIN];
      build_obs(o);
      if (obs_p) {
        flush_rows(o, obs_p);
        obs_p += TE * (N * D);
      }
      pack_operands(o, b1);
    }
    // ---- policy: four 16-row tiles per wavefront
    if constexpr (!UNIFORM) {
      // (a 48-row wavefront has three tiles: the branch is uniform over the wavefront)
      [[maybe_unused]] float value = 0.0f;
      if constexpr (AC) {   // the critic first, through the same stage: its one output is column 0
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (c < 3 || wave_count == 64) policy_tile<N, H>(csm, cbias, b1[c], stage + c * 16 * 5, lane);
        wave_sync();
        value = stage[lane * 5];
        wave_sync();
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (c < 3 || wave_count == 64) policy_tile<N, H>(wsm, bias, b1[c], stage + c * 16 * 5, lane);
      wave_sync();
      float z[kNumActions];
#pragma unroll
      for (int k = 0; k < kNumActions; ++k) z[k] = stage[lane * 5 + k];
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
          if (valid) value_base[row_off] = value;
          value_base += TE * N;
        }
        wave_sync();   // the stages are rewritten by the next step's tiles
      }
    }
    if (act_base) {
      if (valid) act_base[row_off] = uint8_t(act);
      act_base += TE * N;
    }

    // ---- transition of this lane's agent
    float fx = A.ph.accel * action_dir_x(act);
    float fy = A.ph.accel * action_dir_y(act);
    // the k-th OTHER agent is agent k (k < i) or k + 1: N - 1 evaluations, ascending agent order
#pragma unroll
    for (int k = 0; k < N - 1; ++k) {
      const float2 q = cur[k + (k >= i ? 1 : 0)];
      const float dx = px - q.x;
      const float dy = py - q.y;
      const float kf = contact_factor(dx, dy, A.ph);
      fx = fmaf(kf, dx, fx);
      fy = fmaf(kf, dy, fy);
    }
    px = fmaf(vx, A.ph.dt, px);
    py = fmaf(vy, A.ph.dt, py);
    vx = fmaf(fx, A.ph.dt_over_mass, vx * A.ph.keep);
    vy = fmaf(fy, A.ph.dt_over_mass, vy * A.ph.keep);
    float2* np = newpos + (t & 1) * ROWS;
    if (active) np[tid] = make_float2(px, py);
    // (C) new positions of this step and coverage distances of the previous one are visible
    group_barrier(arrived, uint32_t(GW) * uint32_t(t + 1), lane, A.fault, A.barrier_polls);

    // reward of the previous step: sum of its N per-landmark distances
    if (t > 0) store_reward((t - 1) & 1);
    float qx[N], qy[N];
#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float2 p = np[el * N + a];
      qx[a] = p.x;
      qy[a] = p.y;
    }
    cur = np + el * N;
    if constexpr (PER_AGENT) {
      overlaps = 0;
#pragma unroll
      for (int a = 0; a < N; ++a) {
        if (a != i) {
          const float dx = px - qx[a], dy = py - qy[a];
          overlaps += fmaf(dx, dx, dy * dy) < A.ph.two_r_sq ? 1u : 0u;
        }
      }
    }
    // coverage term of landmark i: min over agents of the distance to it (post-step, pre-reset)
    {
      float best2 = INFINITY;
#pragma unroll
      for (int a = 0; a < N; ++a) {
        const float dx = qx[a] - mylx, dy = qy[a] - myly;
        best2 = fminf(best2, fmaf(dx, dx, dy * dy));
      }
      if (active) dminbuf[(t & 1) * ROWS + tid] = hw_sqrt(best2);
    }
    ep += 1;
    const bool done = ep >= A.ph.max_ep;
    if (done_base) {
      if (env_writer) done_base[gc] = done ? 1 : 0;
      done_base += TE;
    }
    if (done) {
      // new episode keyed by step + 1; every lane regenerates the whole env (rare: 1 step in
      // max_ep) and writes all its positions and landmarks: the lanes of an env store identical
      // values, and a lane reads them back only after its own stores (the exchange buffer itself
      // is left alone: slower lanes of the env may still be reading the pre-reset positions).
      // The empty asm keeps the compiler from hoisting the env-dependent first Philox round of
      // all 2N streams out of the step loop.
      uint32_t env_r = env;
      asm volatile("" : "+v"(env_r));
#pragma unroll
      for (int a = 0; a < N; ++a) {
        const uint4 w = philox4x32_10(env_r, step + 1u, uint32_t(a), kTagResetPos, A.seed, run);
        const float2 p = make_float2(word_to_position(w.x), word_to_position(w.y));
        if (active) respos[el * N + a] = p;
        const uint4 wl = philox4x32_10(env_r, step + 1u, uint32_t(N + a), kTagResetPos, A.seed, run);
        const float2 lm = make_float2(word_to_position(wl.x), word_to_position(wl.y));
        if (active) lmbuf[el * N + a] = lm;
        if (a == i) { px = p.x; py = p.y; mylx = lm.x; myly = lm.y; }
      }
      cur = respos + el * N;
      vx = vy = 0.0f;
      ep = 0;
    }
  }
  group_barrier(arrived, uint32_t(GW) * uint32_t(A.T + 1), lane, A.fault, A.barrier_polls);  // coverage distances of the last step
  store_reward((A.T - 1) & 1);
  if (A.last_obs) {
    float o[KIN];
    build_obs(o);
    flush_rows(o, A.last_obs + wave_row0);
  }
  if constexpr (AC) {
    if (A.last_value) {   // value of the observation after the last step
      float o[KIN];
      build_obs(o);
      bf16x8 b1[4][S::S1];
      pack_operands(o, b1);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (c < 3 || wave_count == 64) policy_tile<N, H>(csm, cbias, b1[c], stage + c * 16 * 5, lane);
      wave_sync();
      if (valid) A.last_value[row_off] = stage[lane * 5];
    }
  }

  // ---- state back to HBM
  if (valid) {
    A.st.pos_a[(0 * N + i) * TE + g] = px;
    A.st.pos_a[(1 * N + i) * TE + g] = py;
    A.st.vel_a[(0 * N + i) * TE + g] = vx;
    A.st.vel_a[(1 * N + i) * TE + g] = vy;
    A.st.pos_l[(0 * N + i) * TE + g] = mylx;
    A.st.pos_l[(1 * N + i) * TE + g] = myly;
    if (i == 0) A.st.ep_step[g] = ep;
  }
}

template <int N, int H>
hipError_t pack_impl(PolicyBuffers& pb, int R, const float* W1, const float* b1, const float* W2,
                     const float* b2, const float* W3, const float* b3, int nout, hipStream_t s) {
  using S = Shape<N, H>;
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * S::RUN_BYTES); e != hipSuccess) return e;
  const int total = int(S::RUN_BYTES / 2);  // upper bound on elements of one run
  dim3 grid(cdiv(total, 256), R);
  hipLaunchKernelGGL((pack_policy_kernel<N, H>), grid, dim3(256), 0, s,
                     static_cast<uint8_t*>(pb.packed), W1, b1, W2, b2, W3, b3, nout);
  return hipGetLastError();
}

template <int N, int H, int EB, int MINW, bool PER_AGENT, bool UNIFORM = false, bool AC = false>
hipError_t rollout_impl(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const void* critic = nullptr) {
  using M = Smem<N, H, EB, UNIFORM, AC>;
  auto kern = rollout_policy_kernel<N, H, EB, MINW, PER_AGENT, UNIFORM, AC>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (hipError_t e = allow_lds(reinterpret_cast<const void*>(kern), M::TOTAL, lds_allowed); e != hipSuccess) return e;
  const uint32_t groups = (A.TE + EB - 1) / EB;
  const uint32_t per_xcd = (groups + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(RowMap<N, EB, UNIFORM>::WAVES * 64), M::TOTAL, s, A, static_cast<const uint8_t*>(pb.packed),
                     static_cast<const uint8_t*>(critic), int(A.TE != A.E), groups, per_xcd);
  return hipGetLastError();
}

}  // namespace

// General shapes built: (N, H, envs per block, min waves per SIMD), bf16 operands.  The kernel takes any
// agent count (rows of 6N floats leave as 16-byte chunks, 8-byte ones when N is odd) and any width that is
// a multiple of 32; a block is at most four sync groups (the smallest env count whose rows fill whole
// wavefronts: 16 envs with 4 agents, 32 with 6, 8 with 8, 32 with 10, 64 with an odd count).
#define MPE_WIDE_POLICY_CASES(X) \
  X(10, 128, 64, 3) X(10, 64, 64, 3) X(9, 128, 64, 3) X(9, 64, 64, 3) X(8, 128, 32, 3) X(8, 64, 32, 3) X(7, 128, 64, 3) \
  X(7, 64, 64, 3) X(6, 128, 64, 3) X(6, 64, 64, 3) X(5, 128, 64, 3) X(5, 64, 64, 3) X(4, 128, 64, 3) X(4, 64, 64, 3)
// Env-only rollouts that use this kernel's lane-per-agent mapping: 4 and more agents (measured 4.6-5.3 TB/s
// of trajectory writes against 1.8-4.2 TB/s of the env-per-lane kernel, whose lanes each own 6 N^2 floats
// per step); the width is not used there.
#define MPE_WIDE_CASES(X) \
  X(10, 128, 64, 3) X(9, 64, 64, 3) X(8, 64, 32, 3) X(7, 64, 64, 3) X(6, 64, 64, 3) X(5, 64, 64, 3) X(4, 64, 64, 3)

bool wide_supported(int N, int H) {
#define X(N_, H_, EB_, MW_) if (N == N_ && H == H_) return true;
  MPE_WIDE_POLICY_CASES(X)
#undef X
  return false;
}

size_t packed_run_bytes_wide(int N, int H) {
#define X(N_, H_, EB_, MW_) if (N == N_ && H == H_) return Shape<N_, H_>::RUN_BYTES;
  MPE_WIDE_POLICY_CASES(X)
#undef X
  return 0;
}

hipError_t pack_policy_wide(PolicyBuffers& pb, int N, int H, int R, const float* W1, const float* b1,
                            const float* W2, const float* b2, const float* W3, const float* b3, int nout,
                            hipStream_t s) {
#define X(N_, H_, EB_, MW_) if (N == N_ && H == H_) return pack_impl<N_, H_>(pb, R, W1, b1, W2, b2, W3, b3, nout, s);
  MPE_WIDE_POLICY_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

// Env-only rollout (seeded uniform actions) with the lane-per-agent mapping of the wide kernel.
bool uniform_wide_supported(int N) {
#define X(N_, H_, EB_, MW_) if (N == N_) return true;
  MPE_WIDE_CASES(X)
#undef X
  return false;
}

hipError_t launch_rollout_uniform_wide(int N, const RolloutArgs& A, hipStream_t s) {
  const PolicyBuffers none{};
#define X(N_, H_, EB_, MW_)                                                                      \
  if (N == N_)                                                                                   \
    return A.ph.reward_mode == 1 ? rollout_impl<N_, H_, EB_, MW_, true, true>(A, none, s)        \
                                 : rollout_impl<N_, H_, EB_, MW_, false, true>(A, none, s);
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
    return A.ph.reward_mode == 1 ? rollout_impl<N_, H_, EB_, MW_, true>(A, pb, s)                \
                                 : rollout_impl<N_, H_, EB_, MW_, false>(A, pb, s);              \
  }
  MPE_WIDE_POLICY_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

// Actor-critic rollout with the lane-per-agent kernel: policy and critic images both staged per block.
hipError_t launch_rollout_ac_wide(int N, int H, const RolloutArgs& A, const PolicyBuffers& pb,
                                  const PolicyBuffers& critic, hipStream_t s, const char** why) {
#define X(N_, H_, EB_, MW_)                                                                          \
  if (N == N_ && H == H_) {                                                                          \
    if (A.TE != A.E && (A.E % EB_) != 0) {                                                           \
      *why = "with several runs, num_envs per run must be a multiple of the block's env count";      \
      return hipSuccess;                                                                             \
    }                                                                                                \
    return A.ph.reward_mode == 1 ? rollout_impl<N_, H_, EB_, MW_, true, false, true>(A, pb, s, critic.packed)  \
                                 : rollout_impl<N_, H_, EB_, MW_, false, false, true>(A, pb, s, critic.packed); \
  }
  MPE_WIDE_POLICY_CASES(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace mpe
