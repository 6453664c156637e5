// Fused rollout with the recurrent policy of the paper's headline speed figure (Fig. 3: an RNN
// agent on MPE; App. G "Recurrent network": hidden width 128, two fully-connected layers of
// width 128): per agent and step
//     e = tanh(We^T o + be);  r, z, n gates of a GRU on (e, h);  h' = (1 - z) n + z h;
//     y = tanh(Wf^T h' + bf);  logits = Wo^T y + bo;  Gumbel-max;  simple-spread transition.
// bf16 weights and layer inputs (nearest even), fp32 accumulation, gate arithmetic and carried
// state: the contraction runs on the bf16 matrix cores, one instruction per product.
//
// Design.  The network has 240 KB of bf16 weights, more than the 160 KB of LDS, and 236 matrix
// instructions per 16 rows: re-reading the weights per wavefront from L2 would cost ~90 GB per
// rollout.  So the weights are STATIONARY and the activations move: a block is 8 wavefronts around
// 64 envs (64 N agent rows; 32 or 16 envs for small batches); wavefront u owns hidden units 16u..16u+15 of every layer and keeps
// its 24 GRU A-operands (r, z, n gates x input/recurrent x 4 K slices) and its embedding operand
// in registers for the whole rollout (100 of its 256 registers); the small layers' operands
// (second fully-connected layer, logits) sit in LDS.  Activations of all rows go through LDS as
// bf16 rows of 128 (+ 16 bytes of padding per row) in which the rows 4..11 of every 16-row tile hold
// each pair of neighbouring 16-byte pieces swapped (act_piece below): padding and swap together make
// the 16-byte operand reads free of bank conflicts.  Every wavefront reads all K of a row tile
// and writes its own 16 units.  The
// carried state stays in fp32 registers of the owning wavefront (4 values per lane and row tile);
// its bf16 copy for the next product lives in LDS.  Phases of a step, separated by block barriers:
//   embed -> X | gates (reads X, HB) | HB <- h' | fc (reads HB) -> Y=X | logits -> L |
//   agents: sample, move, exchange positions | reward, done, auto-reset, next observation
// (the agent lanes store their fp32 observation rows straight to the trajectory and leave a bf16
// copy in LDS for the embedding).
// The first 64 N threads are also the agents (one lane per agent row) for the environment part.
// The kernel is a template over the scenario of the family (App. B.7): simple spread with 1..10 agents or a
// predator-prey shape; the network phases see only rows, the two agent phases hold the scenario's own
// transition, rewards, reset and observation.  Observations wider than 32 entries (6 and more agents of
// simple spread) enter the embedding as two K slices.
#include "mpe_mlp64.h"
#include "mpe_tag_device.h"

namespace mpe {

namespace {

constexpr int kG = 128;    // hidden width of every layer
constexpr int kAS = 272;   // bytes per activation row in LDS: 128 bf16 + 16 bytes of padding

// LDS access rules of this chip, read off the bank-conflict counter (SQ_LDS_BANK_CONFLICT) on stand-alone
// access patterns, two active lanes at a time:
//   16-byte read:  64 banks of 4 bytes; four passes of 16 lanes: {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31}
//                  and the same two sets + 32;
//   16-byte write: 32 banks; eight passes of 8 consecutive lanes;
//   8-byte write:  32 banks; four passes of 16 consecutive lanes;
//   4-byte read:   32 banks; two passes of 32 consecutive lanes.
// A k-way conflict inside a pass costs k - 1 extra cycles.
//
// Where the 16-byte piece w (= units 8w .. 8w + 7) of row j of a 16-row tile sits inside the row: piece w
// for rows 0..3 and 12..15, piece w ^ 1 for rows 4..11.  Lane (j, gq) reads piece 4 s + gq of row j, so a
// read pass holds rows {0-3, 12-15} at one gq and rows 4..11 at gq ^ 1; with rows 17 pieces apart, piece
// index j + gq (mod 16) would meet twice in every pass (one extra cycle per pass, four per read: what the
// padding alone costs); the swap turns the pass into 16 different pieces.  An exhaustive search over per-row
// XOR masks inside a K slice finds 8 such layouts at this row stride; masks that reach across slices cost
// address registers, which this kernel spills.  The 8-byte writes of a pass are the same 8 bytes of 16
// different rows: with 16-byte-aligned rows they share 8 bank pairs, one extra cycle per pass, whatever
// the layout.
__device__ __forceinline__ int act_piece(int w, int row_in_tile) { return w ^ (((row_in_tile + 4) >> 3) & 1); }

// The observation tile: bf16 rows of 32 columns = four 16-byte pieces, 64 bytes apart, piece q of row
// `row` at position q ^ ((row >> 1) & 3): free of conflicts both for the embedding's 16-byte reads (lane
// (j, gq) reads piece gq of row 16 rt + j) and for the agent lanes' 16-byte writes (lane = row).
// With two K slices per row (observations of 33..64 entries) rows are 160 bytes apart and piece q = 4 s + p
// sits at 4 s + (p ^ ((row >> 2) & 1)): again free of conflicts for both access kinds.
template <int KS>
__device__ __forceinline__ int obs_piece(int q, int row) {
  return KS == 1 ? (q ^ ((row >> 1) & 3)) : (q ^ ((row >> 2) & 1));
}

// The scenario a kernel instance runs: agents N, observation width D, landmarks L.
template <int N_>
struct GruSpread {
  static constexpr int N = N_, D = 6 * N_, L = N_;
  static constexpr bool kTag = false;
  using Shape = TagShape<2, 1, 1>;   // unused
};
template <int N_, int L_, int G_>
struct GruTag {
  using Shape = TagShape<N_, L_, G_>;
  static constexpr int N = N_, D = Shape::D, L = L_;
  static constexpr bool kTag = true;
};

// Packed weight image (bytes).  A operands of v_mfma_f32_16x16x32_bf16: lane (i = lane % 16,
// gq = lane / 16) holds weights [k = 32 s + 8 gq + e][out = 16 u + i], e = 0..7.
struct GruPk {
  static constexpr size_t OFF_EMB = 0;                         // [u 8][s 2][lane 64]  (K = 64 >= obs width)
  static constexpr size_t OFF_GRU = OFF_EMB + 16 * 1024;       // [u 8][gate 3][src 2][s 4][lane 64]
  static constexpr size_t OFF_FC = OFF_GRU + 8 * 24 * 1024;    // [u 8][s 4][lane 64]
  static constexpr size_t OFF_OUT = OFF_FC + 32 * 1024;        // [s 4][lane 64]  (5 outputs padded to 16)
  static constexpr size_t OFF_BIAS = OFF_OUT + 4 * 1024;       // fp32: be, bi_r + bh_r, bi_z + bh_z, bi_n, bh_n, bf [128 each], bo [16]
  static constexpr int BIAS_FLOATS = 6 * kG + 16;
  static constexpr size_t BYTES = OFF_BIAS + size_t(BIAS_FLOATS) * 4;   // one run; runs follow each other
  static_assert(BYTES % 16 == 0, "images of consecutive runs stay 16-byte aligned");
  static constexpr int N_EMB = 8 * 2 * 64 * 8, N_GRU = 8 * 24 * 64 * 8, N_FC = 8 * 4 * 64 * 8, N_OUT = 4 * 64 * 8;
  static constexpr int THREADS = N_EMB + N_GRU + N_FC + N_OUT + BIAS_FLOATS;
};

// One thread per packed bf16 weight or fp32 bias of one run (blockIdx.y).  D = observation width (<= 64).
__global__ void pack_gru_kernel(uint8_t* __restrict__ out, int D, const float* __restrict__ We,
                                const float* __restrict__ be, const float* __restrict__ Wi,
                                const float* __restrict__ bi, const float* __restrict__ Wh,
                                const float* __restrict__ bh, const float* __restrict__ Wf,
                                const float* __restrict__ bf, const float* __restrict__ Wo,
                                const float* __restrict__ bo) {
  const size_t run = blockIdx.y;
  out += run * GruPk::BYTES;
  We += run * size_t(D) * kG;
  be += run * kG;
  Wi += run * size_t(kG) * 3 * kG;
  bi += run * 3 * kG;
  Wh += run * size_t(kG) * 3 * kG;
  bh += run * 3 * kG;
  Wf += run * size_t(kG) * kG;
  bf += run * kG;
  Wo += run * size_t(kG) * kNumActions;
  bo += run * kNumActions;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < GruPk::N_EMB) {
    const int e = idx % 8, lane = (idx / 8) % 64, sl = (idx / 512) % 2, u = idx / 1024;
    const int k = 32 * sl + 8 * (lane / 16) + e, o = 16 * u + lane % 16;
    reinterpret_cast<uint16_t*>(out + GruPk::OFF_EMB)[idx] = f32_to_bf16_rne(k < D ? We[size_t(k) * kG + o] : 0.0f);
    return;
  }
  idx -= GruPk::N_EMB;
  if (idx < GruPk::N_GRU) {
    const int e = idx % 8, lane = (idx / 8) % 64;
    int rest = idx / 512;
    const int s = rest % 4; rest /= 4;
    const int src = rest % 2; rest /= 2;
    const int gate = rest % 3, u = rest / 3;
    const int k = 32 * s + 8 * (lane / 16) + e, col = gate * kG + 16 * u + lane % 16;
    const float* W = src == 0 ? Wi : Wh;
    reinterpret_cast<uint16_t*>(out + GruPk::OFF_GRU)[idx] = f32_to_bf16_rne(W[size_t(k) * 3 * kG + col]);
    return;
  }
  idx -= GruPk::N_GRU;
  if (idx < GruPk::N_FC) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % 4, u = idx / 2048;
    const int k = 32 * s + 8 * (lane / 16) + e;
    reinterpret_cast<uint16_t*>(out + GruPk::OFF_FC)[idx] = f32_to_bf16_rne(Wf[size_t(k) * kG + 16 * u + lane % 16]);
    return;
  }
  idx -= GruPk::N_FC;
  if (idx < GruPk::N_OUT) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = idx / 512;
    const int k = 32 * s + 8 * (lane / 16) + e, o = lane % 16;
    reinterpret_cast<uint16_t*>(out + GruPk::OFF_OUT)[idx] =
        f32_to_bf16_rne(o < kNumActions ? Wo[size_t(k) * kNumActions + o] : 0.0f);
    return;
  }
  idx -= GruPk::N_OUT;
  if (idx < GruPk::BIAS_FLOATS) {
    float v;
    if (idx < kG) v = be[idx];
    else if (idx < 2 * kG) v = bi[idx - kG] + bh[idx - kG];               // r
    else if (idx < 3 * kG) v = bi[idx - kG] + bh[idx - kG];               // z (columns 128..255)
    else if (idx < 4 * kG) v = bi[idx - kG];                              // n, input part (columns 256..383)
    else if (idx < 5 * kG) v = bh[idx - 2 * kG];                          // n, recurrent part
    else if (idx < 6 * kG) v = bf[idx - 5 * kG];
    else v = (idx - 6 * kG) < kNumActions ? bo[idx - 6 * kG] : 0.0f;
    reinterpret_cast<float*>(out + GruPk::OFF_BIAS)[idx] = v;
  }
}

// Packed critic head of the recurrent actor-critic (bytes, per run): the second fully-connected layer of the
// critic as A operands, [u 8][s 4][lane 64] like the actor's, then fp32: bc [128], wv [128] (rounded to
// bf16), bv [1] and padding.
struct GruCriticPk {
  static constexpr size_t OFF_FC = 0;
  static constexpr size_t OFF_TAIL = 32 * 1024;
  static constexpr int TAIL_FLOATS = 2 * kG + 4;
  static constexpr size_t BYTES = OFF_TAIL + size_t(TAIL_FLOATS) * 4;
  static_assert(BYTES % 16 == 0, "images of consecutive runs stay 16-byte aligned");
  static constexpr int N_FC = 8 * 4 * 64 * 8;
  static constexpr int THREADS = N_FC + TAIL_FLOATS;
};

__global__ void pack_gru_critic_kernel(uint8_t* __restrict__ out, const float* __restrict__ Wc, const float* __restrict__ bc,
                                       const float* __restrict__ wv, const float* __restrict__ bv) {
  const size_t run = blockIdx.y;
  out += run * GruCriticPk::BYTES;
  Wc += run * size_t(kG) * kG;
  bc += run * kG;
  wv += run * kG;
  bv += run;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < GruCriticPk::N_FC) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % 4, u = idx / 2048;
    const int k = 32 * s + 8 * (lane / 16) + e;
    reinterpret_cast<uint16_t*>(out + GruCriticPk::OFF_FC)[idx] = f32_to_bf16_rne(Wc[size_t(k) * kG + 16 * u + lane % 16]);
    return;
  }
  idx -= GruCriticPk::N_FC;
  if (idx < GruCriticPk::TAIL_FLOATS) {
    float v = 0.0f;
    if (idx < kG) v = bc[idx];
    else if (idx < 2 * kG) v = __uint_as_float(uint32_t(f32_to_bf16_rne(wv[idx - kG])) << 16);
    else if (idx == 2 * kG) v = bv[0];
    reinterpret_cast<float*>(out + GruCriticPk::OFF_TAIL)[idx] = v;
  }
}

constexpr size_t up16(size_t x) { return (x + 15) & ~size_t(15); }

// AC: the actor-critic rollout: the critic head's tail (bc, wv, bv) and, per wavefront, the partial value of
// every row (summed by the row's agent lane in a fixed order, so results do not depend on timing).
template <typename Scn, int EB = 64, bool AC = false>
struct GruSmem {
  static constexpr int N = Scn::N;
  static constexpr int B = EB * N, D = Scn::D, NT = B / 16;     // rows, obs width, 16-row tiles
  static constexpr int KS = D <= 32 ? 1 : 2;                    // K slices of the embedding
  static_assert(B % 16 == 0 && EB <= 64 && D <= 64 && D % 2 == 0, "whole row tiles; at most two K slices");
  // bf16 observation tile, 32 KS columns per row (zero beyond D); after the embedding it is dead, and the
  // logits of the same step, [5][B] floats (action-major: the agent lanes read consecutive words), are
  // stored in its place
  static constexpr int OS = KS == 1 ? 64 : 160;
  static constexpr size_t OBS_BYTES = size_t(B) * OS;
  static constexpr size_t LOGIT_BYTES = size_t(B) * kNumActions * 4;
  static constexpr size_t OFF_OBS = 0;
  static constexpr size_t OFF_X = up16(OBS_BYTES > LOGIT_BYTES ? OBS_BYTES : LOGIT_BYTES);   // e, later y
  static constexpr size_t OFF_HB = OFF_X + size_t(B) * kAS;                                  // bf16 copy of h
  static constexpr size_t OFF_FCW = OFF_HB + size_t(B) * kAS;
  static constexpr size_t OFF_OUTW = OFF_FCW + 32 * 1024;
  static constexpr size_t OFF_BIAS = OFF_OUTW + 4 * 1024;
  // [B] new positions (float2); predator-prey: new position and velocity (float4)
  static constexpr size_t OFF_XCH = up16(OFF_BIAS + size_t(GruPk::BIAS_FLOATS) * 4);
  static constexpr size_t OFF_DONE = OFF_XCH + size_t(B) * (Scn::kTag ? 16 : 8);             // [64] bytes
  static constexpr size_t OFF_CTAIL = OFF_DONE + 64;                                         // AC: bc, wv, bv
  static constexpr size_t TOTAL = OFF_CTAIL + (AC ? size_t(GruCriticPk::TAIL_FLOATS) * 4 : 0);
  // AC: the partial values, [8][B] floats, live behind the logits in the dead observation tile (written in the
  // second-layer phase, read by the agent lanes before they write the next observation)
  static constexpr size_t OFF_VPART = OFF_OBS + up16(LOGIT_BYTES);
  static_assert(!AC || OFF_VPART + size_t(8) * B * 4 <= OFF_X, "partial values fit the observation tile");
  static_assert(TOTAL <= 160 * 1024, "LDS");
};

__device__ __forceinline__ float fast_sigmoid(float x) { return hw_rcp(1.0f + hw_exp2(-kLog2e * x)); }

__device__ __forceinline__ uint2 pack4_bf16(float a, float b, float c, float d) {
  return make_uint2(pack_bf16_rne(a, b), pack_bf16_rne(c, d));
}

// EB = envs per block: 64, or 32 / 16 for small batches (every phase of a step is a loop over the block's
// 16-row tiles, so the step latency of a block, which is the time of a rollout while every block has a CU
// to itself, falls with its rows) and for the shapes whose activations would not fit the LDS otherwise.
// AC = the actor-critic rollout (packed_critic = the head of pack_gru_critic): per step also the critic's second
// layer on the new carried state and the log-probability of the sampled action, and, when a bootstrap value
// is asked for, one more pass of the network phases after the last step that writes nothing else.
template <typename Scn, int EB, bool AC>
__global__ __launch_bounds__(512) void rollout_gru_kernel(TagArgs TA, const uint8_t* __restrict__ packed,
                                                          const uint8_t* __restrict__ packed_critic,
                                                          float* __restrict__ hidden, int per_run_weights,
                                                          uint32_t groups, uint32_t groups_per_xcd) {
  using M = GruSmem<Scn, EB, AC>;
  using TS = typename Scn::Shape;                      // predator-prey only
  constexpr bool kTag = Scn::kTag;
  constexpr int N = Scn::N, L = Scn::L, B = M::B, D = M::D, NT = M::NT, KS = M::KS;
  constexpr int G = kTag ? TS::G : 1, NA = kTag ? TS::A : 0;   // good agents, adversaries
  const RolloutArgs& A = TA.r;
  [[maybe_unused]] const TagPhys& tg = TA.tg;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* otile = smem + M::OFF_OBS;
  float* logits = reinterpret_cast<float*>(smem + M::OFF_OBS);
  uint8_t* xbuf = smem + M::OFF_X;
  uint8_t* hbuf = smem + M::OFF_HB;
  const bf16x8* fcw0 = reinterpret_cast<const bf16x8*>(smem + M::OFF_FCW);
  const bf16x8* outw0 = reinterpret_cast<const bf16x8*>(smem + M::OFF_OUTW);
  const float* bias0 = reinterpret_cast<const float*>(smem + M::OFF_BIAS);
  [[maybe_unused]] float2* xch2 = reinterpret_cast<float2*>(smem + M::OFF_XCH);
  [[maybe_unused]] float4* xch4 = reinterpret_cast<float4*>(smem + M::OFF_XCH);
  uint8_t* donef = smem + M::OFF_DONE;
  [[maybe_unused]] const float* ctail0 = reinterpret_cast<const float*>(smem + M::OFF_CTAIL);
  [[maybe_unused]] float* vpart = reinterpret_cast<float*>(smem + M::OFF_VPART);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int u = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront = owned unit tile
  const int j = lane & 15, gq = lane >> 4;
  // Byte offsets of this lane inside a tile of 16 activation rows (every row it touches is row j of its
  // tile): where it writes its 4 units 16 u + 4 gq .. + 3 (8 bytes: half gq & 1 of piece 2 u + gq / 2), and
  // where it reads piece gq of K slice 0 (slice s is 64 s bytes further).  Two values per lane for the whole
  // rollout; tile and slice offsets are constants of the unrolled loops and go into the instructions.
  const int wr_off = j * kAS + 16 * act_piece(2 * u + (gq >> 1), j) + 8 * (gq & 1);
  const int rd_off = j * kAS + 16 * act_piece(gq, j);
  constexpr int kTile = 16 * kAS;   // bytes of one tile of 16 activation rows
  const size_t TE = A.TE;
  const uint32_t grp = (blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3);
  if (grp >= groups) return;  // whole block, before any barrier
  const size_t g0 = size_t(grp) * EB;
  const size_t left = TE - g0;
  const int nvalid = left < size_t(EB) ? int(left) : EB;   // valid envs of this block
  const int vrows = nvalid * N;                            // valid agent rows
  if (per_run_weights) packed += size_t(uint32_t(g0) / A.E) * GruPk::BYTES;   // the run of this block's envs
  if constexpr (AC) {
    if (per_run_weights) packed_critic += size_t(uint32_t(g0) / A.E) * GruCriticPk::BYTES;
  }

  // ---- stationary operands: this wavefront's GRU and embedding tiles in registers; the small
  // layers and all biases in LDS
  bf16x8 wg[3][2][4];
#pragma unroll
  for (int gate = 0; gate < 3; ++gate)
#pragma unroll
    for (int src = 0; src < 2; ++src)
#pragma unroll
      for (int s = 0; s < 4; ++s)
        wg[gate][src][s] = reinterpret_cast<const bf16x8*>(packed + GruPk::OFF_GRU)[(((u * 3 + gate) * 2 + src) * 4 + s) * 64 + lane];
  bf16x8 we[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) we[s] = reinterpret_cast<const bf16x8*>(packed + GruPk::OFF_EMB)[(u * 2 + s) * 64 + lane];
  {
    const uint4* src = reinterpret_cast<const uint4*>(packed + GruPk::OFF_FC);
    uint4* dst = reinterpret_cast<uint4*>(smem + M::OFF_FCW);
    for (int k = tid; k < (32 + 4) * 1024 / 16; k += 512) dst[k] = src[k];      // FC and OUT are adjacent in both
    const float* bsrc = reinterpret_cast<const float*>(packed + GruPk::OFF_BIAS);
    float* bdst = reinterpret_cast<float*>(smem + M::OFF_BIAS);
    for (int k = tid; k < GruPk::BIAS_FLOATS; k += 512) bdst[k] = bsrc[k];
    if (tid < 64) donef[tid] = 0;
    if constexpr (AC) {
      const float* csrc = reinterpret_cast<const float*>(packed_critic + GruCriticPk::OFF_TAIL);
      float* cdst = reinterpret_cast<float*>(smem + M::OFF_CTAIL);
      for (int k = tid; k < GruCriticPk::TAIL_FLOATS; k += 512) cdst[k] = csrc[k];
    }
  }

  // ---- carried state of this wavefront's units: hreg[rt][r] = h[row 16 rt + j][unit 16 u + 4 gq + r]
  float hreg[NT][4];
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    const int row = 16 * rt + j;
    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (row < vrows) v = *reinterpret_cast<const f32x4*>(hidden + (g0 * N + row) * kG + 16 * u + 4 * gq);
#pragma unroll
    for (int r = 0; r < 4; ++r) hreg[rt][r] = v[r];
    *reinterpret_cast<uint2*>(hbuf + rt * kTile + wr_off) = pack4_bf16(v[0], v[1], v[2], v[3]);
  }

  // ---- agents: the first B threads, one lane per agent row
  const bool agent = tid < B;
  const int el = tid / N, i = tid - el * N;          // env within block, agent (agent lanes only)
  const size_t g = g0 + el;
  const bool valid = agent && g < TE;
  const uint32_t gc = valid ? uint32_t(g) : uint32_t(g0);
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;
  float px = 0.0f, py = 0.0f, vx = 0.0f, vy = 0.0f;
  // all agents' positions and the landmarks of this lane's env; predator-prey: the good agents' velocities
  float qx[N], qy[N], lx[L + 1], ly[L + 1];
  [[maybe_unused]] float gvx[G], gvy[G];
  int32_t ep = 0;
#pragma unroll
  for (int a = 0; a < N; ++a) qx[a] = qy[a] = 0.0f;
#pragma unroll
  for (int k = 0; k < L + 1; ++k) lx[k] = ly[k] = 0.0f;
#pragma unroll
  for (int k = 0; k < G; ++k) gvx[k] = gvy[k] = 0.0f;
  if (valid) {
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
    if constexpr (kTag) {
#pragma unroll
      for (int k = 0; k < G; ++k) {
        gvx[k] = A.st.vel_a[(0 * N + NA + k) * TE + g];
        gvy[k] = A.st.vel_a[(1 * N + NA + k) * TE + g];
      }
    }
    vx = A.st.vel_a[(0 * N + i) * TE + g];
    vy = A.st.vel_a[(1 * N + i) * TE + g];
    ep = A.st.ep_step[g];
  }
#pragma unroll
  for (int a = 0; a < N; ++a) {
    if (a == i) { px = qx[a]; py = qy[a]; }
  }
  // predator-prey: the constants of this lane's role
  [[maybe_unused]] TagRole me{};
  if constexpr (kTag) me = tag_role<TS>(i, tg);

  // Observation row of this lane from the registers above: bf16 (nearest even) into the LDS tile
  // for the embedding, fp32 to `dst` (this lane's row of a trajectory slice, may be null).
  auto write_obs_row = [&](float* dst) {
    float o[32 * KS];
#pragma unroll
    for (int c = 0; c < 32 * KS; ++c) o[c] = 0.0f;
    if constexpr (kTag) {
      tag_obs_regs<TS>(o, i, px, py, vx, vy, qx, qy, lx, ly, gvx, gvy);
    } else {
      o[0] = vx; o[1] = vy; o[2] = px; o[3] = py;
#pragma unroll
      for (int l = 0; l < N; ++l) { o[4 + 2 * l] = lx[l] - px; o[5 + 2 * l] = ly[l] - py; }
      // the k-th OTHER agent is agent k (k < i) or k + 1, ascending
#pragma unroll
      for (int k = 0; k < N - 1; ++k) {
        const bool up = k >= i;
        o[4 + 2 * N + 2 * k] = (up ? qx[k + 1] : qx[k]) - px;
        o[5 + 2 * N + 2 * k] = (up ? qy[k + 1] : qy[k]) - py;
      }
    }
    u32x4* row = reinterpret_cast<u32x4*>(otile + tid * M::OS);
#pragma unroll
    for (int q = 0; q < 4 * KS; ++q) {
      u32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = pack_bf16_rne(o[8 * q + 2 * e], o[8 * q + 2 * e + 1]);
      row[obs_piece<KS>(q, tid)] = v;
    }
    if (dst && valid) {
#pragma unroll
      for (int c = 0; c < D / 2; ++c) reinterpret_cast<float2*>(dst)[c] = make_float2(o[2 * c], o[2 * c + 1]);
    }
  };
  const size_t slice = TE * size_t(N * D);                               // floats per time slice
  float* obs_row = A.obs_traj ? A.obs_traj + (size_t(gc) * N + i) * D : nullptr;   // this lane's row, slot 0
  float* last_row = A.last_obs ? A.last_obs + (size_t(gc) * N + i) * D : nullptr;
  if (agent) write_obs_row(obs_row);
  __syncthreads();   // staged weights, biases, HB, first observation

  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  const size_t row_off = size_t(gc) * N + i;
  const bool env_writer = valid && i == 0;
  const bool per_agent_reward = kTag || A.ph.reward_mode == 1;
  uint32_t step = A.abs_step;
  [[maybe_unused]] float* logp_base = A.logp_traj;
  [[maybe_unused]] float* value_base = A.value_traj;

  // The carried state back to HBM (cleared where the last step ended an episode).
  auto store_hidden = [&]() {
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const int row = 16 * rt + j;
      if (row < vrows) {
        const bool fresh = donef[row / N] != 0;
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = fresh ? 0.0f : hreg[rt][r];
        *reinterpret_cast<f32x4*>(hidden + (g0 * N + row) * kG + 16 * u + 4 * gq) = v;
      }
    }
  };
  // This row's value: the critic head's output bias plus the eight wavefronts' partial sums, in a fixed order.
  [[maybe_unused]] auto row_value = [&]() {
    float v = ctail0[2 * kG];
#pragma unroll
    for (int w8 = 0; w8 < 8; ++w8) v += vpart[w8 * B + tid];
    return v;
  };

  // Actor-critic with a bootstrap value: one more pass of the network over the observation after the last
  // step, on the carried state as it stands; that pass writes nothing back (the state has been stored by then).
  const bool bootstrap = AC && A.last_value != nullptr;
  const int passes = A.T + (bootstrap ? 1 : 0);
  for (int t = 0; t < passes; ++t, ++step) {
    const bool extra = AC && t == A.T;
    if (extra) store_hidden();   // the registers of the carried state are free from here on
    // Opaque zero: keeps the step-invariant LDS reads (biases, small-layer operands) inside the step
    // loop; hoisted out of it they would pin ~40 registers for the whole rollout.
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    const float* bias = bias0 + zero;
    const bf16x8* fcw = fcw0 + zero;
    const bf16x8* outw = outw0 + zero;
    // ---- embedding: e = tanh(We^T o + be), this wavefront's 16 units of every row -> X
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const int row = 16 * rt + j;
      f32x4 acc = *reinterpret_cast<const f32x4*>(bias + 16 * u + 4 * gq);
#pragma unroll
      for (int s = 0; s < KS; ++s)
        acc = MPE_MFMA_BF(we[s], *reinterpret_cast<const bf16x8*>(otile + row * M::OS + 16 * obs_piece<KS>(4 * s + gq, j)), acc);
      *reinterpret_cast<uint2*>(xbuf + rt * kTile + wr_off) =
          pack4_bf16(fast_tanh(acc[0]), fast_tanh(acc[1]), fast_tanh(acc[2]), fast_tanh(acc[3]));
    }
    __syncthreads();   // X complete; the observation tile has been read

    // ---- gates and new state of this wavefront's units (reads X and HB of all units)
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const int row = 16 * rt + j;
      // the env finished an episode in the last step: h = 0 (its HB row was cleared by its agent lane)
      const bool fresh = donef[row / N] != 0;
      f32x4 ar = *reinterpret_cast<const f32x4*>(bias + 1 * kG + 16 * u + 4 * gq);
      f32x4 az = *reinterpret_cast<const f32x4*>(bias + 2 * kG + 16 * u + 4 * gq);
      f32x4 ani = *reinterpret_cast<const f32x4*>(bias + 3 * kG + 16 * u + 4 * gq);
      f32x4 anh = *reinterpret_cast<const f32x4*>(bias + 4 * kG + 16 * u + 4 * gq);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 bx = *reinterpret_cast<const bf16x8*>(xbuf + rt * kTile + 64 * s + rd_off);
        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(hbuf + rt * kTile + 64 * s + rd_off);
        // dependent accumulations three instructions apart
        ar = MPE_MFMA_BF(wg[0][0][s], bx, ar);
        az = MPE_MFMA_BF(wg[1][0][s], bx, az);
        ani = MPE_MFMA_BF(wg[2][0][s], bx, ani);
        ar = MPE_MFMA_BF(wg[0][1][s], bh, ar);
        az = MPE_MFMA_BF(wg[1][1][s], bh, az);
        anh = MPE_MFMA_BF(wg[2][1][s], bh, anh);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float h = fresh ? 0.0f : hreg[rt][r];
        const float rr = fast_sigmoid(ar[r]);
        const float zz = fast_sigmoid(az[r]);
        const float nn = fast_tanh(fmaf(rr, anh[r], ani[r]));
        hreg[rt][r] = fmaf(zz, h - nn, nn);      // (1 - z) n + z h
      }
    }
    __syncthreads();   // every wavefront has read the old HB
#pragma unroll
    for (int rt = 0; rt < NT; ++rt)
      *reinterpret_cast<uint2*>(hbuf + rt * kTile + wr_off) =
          pack4_bf16(hreg[rt][0], hreg[rt][1], hreg[rt][2], hreg[rt][3]);
    __syncthreads();   // HB = bf16(h')

    // ---- second fully-connected layer: y = tanh(Wf^T h' + bf) -> X (e is dead); actor-critic: also the
    // critic's second layer yc = tanh(Wc^T h' + bc) and this wavefront's share of value = wv^T yc + bv
    {
      bf16x8 wf[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) wf[s] = fcw[(u * 4 + s) * 64 + lane];
#pragma unroll
      for (int rt = 0; rt < NT; ++rt) {
        f32x4 acc = *reinterpret_cast<const f32x4*>(bias + 5 * kG + 16 * u + 4 * gq);
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc = MPE_MFMA_BF(wf[s], *reinterpret_cast<const bf16x8*>(hbuf + rt * kTile + 64 * s + rd_off), acc);
        *reinterpret_cast<uint2*>(xbuf + rt * kTile + wr_off) =
            pack4_bf16(fast_tanh(acc[0]), fast_tanh(acc[1]), fast_tanh(acc[2]), fast_tanh(acc[3]));
      }
    }
    if constexpr (AC) {
      // a pass of its own over the row tiles (the state's bf16 copy is read again), so that the actor's and the
      // critic's operands are not live together; the critic's come from global memory every step (32 KB per
      // run, cache-resident): the LDS has no room for them beside the actor's
      const bf16x8* cw = reinterpret_cast<const bf16x8*>(packed_critic + GruCriticPk::OFF_FC) + zero;
      bf16x8 wc[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) wc[s] = cw[(u * 4 + s) * 64 + lane];
      const float* ctail = ctail0 + zero;
      const f32x4 bcv = *reinterpret_cast<const f32x4*>(ctail + 16 * u + 4 * gq);
      const f32x4 wvv = *reinterpret_cast<const f32x4*>(ctail + kG + 16 * u + 4 * gq);
#pragma unroll
      for (int rt = 0; rt < NT; ++rt) {
        f32x4 accc = bcv;
#pragma unroll
        for (int s = 0; s < 4; ++s)
          accc = MPE_MFMA_BF(wc[s], *reinterpret_cast<const bf16x8*>(hbuf + rt * kTile + 64 * s + rd_off), accc);
        // yc enters the last product rounded to bf16; lane (j, gq) holds units 16 u + 4 gq .. + 3 of row j
        const uint2 yc = pack4_bf16(fast_tanh(accc[0]), fast_tanh(accc[1]), fast_tanh(accc[2]), fast_tanh(accc[3]));
        float pv = __uint_as_float(yc.x << 16) * wvv[0];
        pv = fmaf(__uint_as_float(yc.x & 0xFFFF0000u), wvv[1], pv);
        pv = fmaf(__uint_as_float(yc.y << 16), wvv[2], pv);
        pv = fmaf(__uint_as_float(yc.y & 0xFFFF0000u), wvv[3], pv);
        pv += __shfl_xor(pv, 16);
        pv += __shfl_xor(pv, 32);
        if (gq == 0) vpart[u * B + 16 * rt + j] = pv;
      }
    }
    __syncthreads();   // Y complete (and the partial values)
    if constexpr (AC) {
      if (extra) {   // bootstrap pass: the value of the observation after the last step, nothing else
        if (valid) A.last_value[row_off] = row_value();
        break;
      }
    }

    // ---- logits of row tiles u, u + 8 -> L (in place of the observation tile)
    for (int rt = u; rt < NT; rt += 8) {
      const int row = 16 * rt + j;
      f32x4 acc = *reinterpret_cast<const f32x4*>(bias + 6 * kG + 4 * gq);
#pragma unroll
      for (int s = 0; s < 4; ++s)
        acc = MPE_MFMA_BF(outw[s * 64 + lane], *reinterpret_cast<const bf16x8*>(xbuf + rt * kTile + 64 * s + rd_off), acc);
      if (gq == 0) {                                                        // outputs 0..3
#pragma unroll
        for (int r = 0; r < 4; ++r) logits[r * B + row] = acc[r];
      } else if (gq == 1) {
        logits[4 * B + row] = acc[0];                                       // output 4
      }
    }
    __syncthreads();   // L complete

    // ---- agents: sample, store, move
    if (agent) {
      float z[kNumActions];
#pragma unroll
      for (int k = 0; k < kNumActions; ++k) z[k] = logits[k * B + tid];
      const uint32_t act = gumbel_argmax(z, A.seed, run, env, step, uint32_t(i));
      if (act_base && valid) act_base[row_off] = uint8_t(act);
      if constexpr (AC) {
        // log pi(act | obs) = z_act - max - ln sum exp(z - max); value of the carried state this step produced
        float zmax = z[0], zact = z[0];
#pragma unroll
        for (int k = 1; k < kNumActions; ++k) {
          zmax = fmaxf(zmax, z[k]);
          zact = act == uint32_t(k) ? z[k] : zact;
        }
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < kNumActions; ++k) sum += hw_exp2((z[k] - zmax) * kLog2e);
        if (logp_base && valid) logp_base[row_off] = (zact - zmax) - kLn2 * hw_log2(sum);
        if (value_base && valid) value_base[row_off] = row_value();
      }
      if constexpr (kTag) {
        tag_move<TS>(act, i, me, tg, px, py, vx, vy, qx, qy, lx, ly);
        xch4[tid] = make_float4(px, py, vx, vy);
      } else {
        agent_move<N>(act, i, A.ph, px, py, vx, vy, qx, qy);
        xch2[tid] = make_float2(px, py);
      }
    }
    if (act_base) act_base += TE * N;
    if constexpr (AC) {
      if (logp_base) logp_base += TE * N;
      if (value_base) value_base += TE * N;
    }
    __syncthreads();   // new positions visible; L has been read

    // ---- agents: reward, done, auto-reset, next observation (written over L)
    if (agent) {
      int32_t max_ep;
      if constexpr (kTag) {
#pragma unroll
        for (int a = 0; a < N; ++a) {
          const float4 p = xch4[el * N + a];
          qx[a] = p.x;
          qy[a] = p.y;
          if (a >= NA) {
            gvx[a - NA] = p.z;
            gvy[a - NA] = p.w;
          }
        }
        if (rew_base && valid) rew_base[row_off] = tag_reward<TS>(i, me, tg, px, py, qx, qy);
        max_ep = tg.max_ep;
      } else {
#pragma unroll
        for (int a = 0; a < N; ++a) {
          const float2 p = xch2[el * N + a];
          qx[a] = p.x;
          qy[a] = p.y;
        }
        const float r = coverage_reward(qx, qy, lx, ly);
        if (A.ph.reward_mode == 1) {
          const uint32_t overlaps = overlap_count<N>(i, px, py, qx, qy, A.ph);
          if (rew_base && valid) rew_base[row_off] = mixed_reward(r, overlaps, A.ph);
        } else if (rew_base && env_writer) {
          rew_base[gc] = r;
        }
        max_ep = A.ph.max_ep;
      }
      ep += 1;
      const bool done = ep >= max_ep;
      if (done_base && env_writer) done_base[gc] = done ? 1 : 0;
      if (i == 0) donef[el] = done ? 1 : 0;     // read by the gate phase of the next step
      if (done) {
        // new episode keyed by step + 1; every lane regenerates its whole env (1 step in max_ep)
        uint32_t env_r = env;
        asm volatile("" : "+v"(env_r));
        if constexpr (kTag) {
          tag_draw_positions<TS>(qx, qy, lx, ly, env_r, step + 1u, A.seed, run);
#pragma unroll
          for (int k = 0; k < G; ++k) gvx[k] = gvy[k] = 0.0f;
        } else {
#pragma unroll
          for (int a = 0; a < N; ++a) {
            const uint4 w = philox4x32_10(env_r, step + 1u, uint32_t(a), kTagResetPos, A.seed, run);
            qx[a] = word_to_position(w.x);
            qy[a] = word_to_position(w.y);
            const uint4 wl = philox4x32_10(env_r, step + 1u, uint32_t(N + a), kTagResetPos, A.seed, run);
            lx[a] = word_to_position(wl.x);
            ly[a] = word_to_position(wl.y);
          }
        }
#pragma unroll
        for (int a = 0; a < N; ++a) {
          if (a == i) { px = qx[a]; py = qy[a]; }
        }
        vx = vy = 0.0f;
        ep = 0;
        // the carried state of the new episode is zero: clear this row's bf16 copy (the fp32
        // registers of the owning wavefronts follow the done flag)
#pragma unroll
        for (int q = 0; q < 16; ++q) reinterpret_cast<u32x4*>(hbuf + tid * kAS)[q] = u32x4{0u, 0u, 0u, 0u};
      }
      if (obs_row) obs_row += slice;
      write_obs_row(t + 1 < A.T ? obs_row : last_row);
    }
    if (rew_base) rew_base += per_agent_reward ? TE * N : TE;
    if (done_base) done_base += TE;
    __syncthreads();   // next observation and the done flags complete
  }

  // ---- state back to HBM: the carried state (unless the bootstrap pass has stored it), agents
  if (!bootstrap) store_hidden();
  if (valid) {
    A.st.pos_a[(0 * N + i) * TE + g] = px;
    A.st.pos_a[(1 * N + i) * TE + g] = py;
    A.st.vel_a[(0 * N + i) * TE + g] = vx;
    A.st.vel_a[(1 * N + i) * TE + g] = vy;
    // landmark l is written back by the lane of agent l % N (every lane holds all of them)
#pragma unroll
    for (int l = 0; l < L; ++l) {
      if (l % N == i) {
        A.st.pos_l[(0 * L + l) * TE + g] = lx[l];
        A.st.pos_l[(1 * L + l) * TE + g] = ly[l];
      }
    }
    if (i == 0) A.st.ep_step[g] = ep;
  }
}

template <typename Scn, int EB, bool AC>
hipError_t rollout_gru_blocks(const TagArgs& A, const PolicyBuffers& pb, const void* critic, float* hidden, hipStream_t s) {
  using M = GruSmem<Scn, EB, AC>;
  auto kern = rollout_gru_kernel<Scn, EB, AC>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (hipError_t e = allow_lds(reinterpret_cast<const void*>(kern), M::TOTAL, lds_allowed); e != hipSuccess) return e;
  const uint32_t groups = (A.r.TE + EB - 1) / EB;
  const uint32_t per_xcd = (groups + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(512), M::TOTAL, s, A, static_cast<const uint8_t*>(pb.packed),
                     static_cast<const uint8_t*>(critic), hidden, int(A.r.TE != A.r.E), groups, per_xcd);
  return hipGetLastError();
}

// The largest block (in envs) whose activations fit the LDS: 64 envs for up to 3 agents, 32 envs for up to 6
// agents whose observation fits one K slice, 16 envs otherwise.
template <typename Scn>
constexpr int gru_max_envs() {
  return Scn::N <= 3 ? 64 : ((Scn::N <= 6 && Scn::D <= 32) ? 32 : 16);
}

template <typename Scn, bool AC>
hipError_t rollout_gru_sized(const TagArgs& A, const PolicyBuffers& pb, const void* critic, float* hidden, hipStream_t s) {
  // Smaller blocks while each still gets a CU to itself (measured per 128-step rollout, 3 agents: 16-env
  // blocks 0.57-0.60 ms up to 4,096 envs and 32-env blocks 0.96-1.01 ms up to 8,192 envs against 1.9 ms with
  // 64-env blocks; with more blocks than CUs the largest blocks are the fastest).
  // With one set of weights per run a block must lie inside a run: the largest of 64, 32, 16 that divides
  // the run size bounds the choice.
  constexpr int kMax = gru_max_envs<Scn>();
  const uint32_t cus = compute_units();
  const bool runs = A.r.TE != A.r.E;
  if (kMax == 16 || (A.r.TE + 15) / 16 <= cus || (runs && A.r.E % 32 != 0))
    return rollout_gru_blocks<Scn, 16, AC>(A, pb, critic, hidden, s);
  if constexpr (kMax >= 32) {
    if (kMax == 32 || (A.r.TE + 31) / 32 <= cus || (runs && A.r.E % 64 != 0))
      return rollout_gru_blocks<Scn, 32, AC>(A, pb, critic, hidden, s);
  }
  if constexpr (kMax >= 64) return rollout_gru_blocks<Scn, 64, AC>(A, pb, critic, hidden, s);
  return hipErrorInvalidValue;
}

template <typename Scn>
hipError_t rollout_gru_impl(const TagArgs& A, const PolicyBuffers& pb, const void* critic, float* hidden, hipStream_t s,
                            const char** why) {
  if (A.r.TE != A.r.E && A.r.E % 16 != 0) {
    *why = "with several runs, num_envs per run must be a multiple of 16";
    return hipSuccess;
  }
  // critic: the packed head of the actor-critic rollout (same block shapes: its partial values live in LDS
  // that is dead at that point of the step)
  return critic ? rollout_gru_sized<Scn, true>(A, pb, critic, hidden, s)
                : rollout_gru_sized<Scn, false>(A, pb, nullptr, hidden, s);
}

__global__ void fill_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t k = size_t(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += size_t(gridDim.x) * blockDim.x) p[k] = 0.0f;
}

}  // namespace

void launch_fill_zero(float* p, size_t n, hipStream_t s) {
  if (n == 0) return;
  const size_t blocks = (n + 255) / 256;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(uint32_t(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, p, n);
}

// Simple spread with 1..10 agents and every predator-prey shape that is built; hidden 128, bf16 weights.
#define MPE_GRU_TAG_SHAPES(X) X(4, 2, 1) X(2, 1, 1) X(3, 0, 1) X(6, 2, 2) X(5, 2, 1) X(8, 2, 2) X(10, 3, 2)

bool gru_supported(bool tag, int N, int L, int G, int H, int weight_dtype) {
  if (H != kG || weight_dtype != 1) return false;
  if (!tag) return N >= 1 && N <= 10;
#define X(n, l, g) if (N == n && L == l && G == g) return true;
  MPE_GRU_TAG_SHAPES(X)
#undef X
  return false;
}

hipError_t pack_policy_gru(PolicyBuffers& pb, int D, int R, const float* We, const float* be, const float* Wi,
                           const float* bi, const float* Wh, const float* bh, const float* Wf, const float* bf,
                           const float* Wo, const float* bo, hipStream_t s) {
  if (D < 1 || D > 64) return hipErrorInvalidValue;
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * GruPk::BYTES); e != hipSuccess) return e;
  hipLaunchKernelGGL(pack_gru_kernel, dim3((GruPk::THREADS + 255) / 256, R), dim3(256), 0, s,
                     static_cast<uint8_t*>(pb.packed), D, We, be, Wi, bi, Wh, bh, Wf, bf, Wo, bo);
  return hipGetLastError();
}

hipError_t pack_gru_critic(PolicyBuffers& pb, int R, const float* Wc, const float* bc, const float* wv, const float* bv,
                           hipStream_t s) {
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * GruCriticPk::BYTES); e != hipSuccess) return e;
  hipLaunchKernelGGL(pack_gru_critic_kernel, dim3((GruCriticPk::THREADS + 255) / 256, R), dim3(256), 0, s,
                     static_cast<uint8_t*>(pb.packed), Wc, bc, wv, bv);
  return hipGetLastError();
}

hipError_t launch_rollout_gru(bool tag, int N, int L, int G, const TagArgs& A, const PolicyBuffers& pb, const void* critic,
                              float* hidden, hipStream_t s, const char** why) {
  if (tag) {
#define X(n, l, g) \
    if (N == n && L == l && G == g) return rollout_gru_impl<GruTag<n, l, g>>(A, pb, critic, hidden, s, why);
    MPE_GRU_TAG_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
  }
  switch (N) {
    case 1: return rollout_gru_impl<GruSpread<1>>(A, pb, critic, hidden, s, why);
    case 2: return rollout_gru_impl<GruSpread<2>>(A, pb, critic, hidden, s, why);
    case 3: return rollout_gru_impl<GruSpread<3>>(A, pb, critic, hidden, s, why);
    case 4: return rollout_gru_impl<GruSpread<4>>(A, pb, critic, hidden, s, why);
    case 5: return rollout_gru_impl<GruSpread<5>>(A, pb, critic, hidden, s, why);
    case 6: return rollout_gru_impl<GruSpread<6>>(A, pb, critic, hidden, s, why);
    case 7: return rollout_gru_impl<GruSpread<7>>(A, pb, critic, hidden, s, why);
    case 8: return rollout_gru_impl<GruSpread<8>>(A, pb, critic, hidden, s, why);
    case 9: return rollout_gru_impl<GruSpread<9>>(A, pb, critic, hidden, s, why);
    case 10: return rollout_gru_impl<GruSpread<10>>(A, pb, critic, hidden, s, why);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mpe
