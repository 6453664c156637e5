// Fused rollout kernel for the headline shape: fp32 policy 6N -> 64 -> 64 -> 5 (N <= 3 agents),
// shared by all agents or one set of weights per run (paper: App. G IPPO table, two tanh layers
// of width 64; Sec. 3.2 parameter sharing; Sec. 4.2 / App. F vmap over whole training runs).
//
// Where the contraction runs.  On gfx950 the fp32 MFMA shares the vector datapath: fp32 matrix
// and fp32 vector peaks are the same number, and measured MFMA-f32 and VALU time add up instead
// of overlapping.  The 16-bit matrix cores are a separate unit, 16x faster per K, and do overlap
// with VALU work.  So every fp32 operand is split EXACTLY into three bf16 terms
//     x = h + m + l,   h = top 16 bits of x, m = top 16 bits of (x - h), l = x - h - m
// (8 + 8 + 8 = 24 significant bits; each difference is exact in fp32) and the product of two
// operands is accumulated in fp32 from the six cross terms of weight >= 2^-16:
//     x*w ~= hh + hm + mh + hl + lh + mm      (dropped: ml + lm + ll <= 2^-23 |x w|)
// i.e. the same operand values as an fp32 GEMM, with a truncation of the order of one fp32
// rounding.  Weights are split once by the pack kernel; activations are split in registers.
//
// Mapping: one lane per agent row; a wavefront owns 64 rows = two pairs of 16-row tiles; each
// A operand (weights, from LDS) is loaded once per pair.  The accumulator layout of
// v_mfma_f32_16x16x32_bf16 (lane (j, gq) holds batch row j and hidden units 16m + 4gq + r) is
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
#include "mpe_policy_common.h"

namespace mpe {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kH = 64;                    // hidden width
constexpr float kPre = 2.0f * kLog2e;     // both tanh layers get pre-activations already times 2*log2(e)

// ------------------------------------------------------------------------------ exact split
// Bit patterns of the three terms as floats whose low 16 bits are zero.
__host__ __device__ __forceinline__ void split3(float x, uint32_t& h, uint32_t& m, uint32_t& l) {
#if defined(__HIP_DEVICE_COMPILE__)
  h = __float_as_uint(x) & 0xFFFF0000u;
  const float r1 = x - __uint_as_float(h);
  m = __float_as_uint(r1) & 0xFFFF0000u;
  l = __float_as_uint(r1 - __uint_as_float(m));
#else
  h = m = l = 0;
  (void)x;
#endif
}
// Pack the high halves of two float bit patterns: low 16 bits <- a, high 16 bits <- b.
__device__ __forceinline__ uint32_t pack_hi16(uint32_t a, uint32_t b) {
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// Packed per-run layout (bytes).  A operands of v_mfma_f32_16x16x32_bf16: lane (i = lane%16,
// gq = lane/16) holds weights [k = 8 gq + e][out = 16 m + i], e = 0..7 (16 bytes), per term.
//   W1A [m 4][combo 2][lane 64]  layer 1 has only 16 inputs, half of the instruction's K = 32, so
//                                 two cross terms share one instruction: K positions 0..15 (lanes
//                                 gq < 2) carry one term of input k' = 8 (gq & 1) + e, positions
//                                 16..31 (gq >= 2) another term of the same inputs.
//                                 combo 0 = (h | m), combo 1 = (h | l)
//   W2A [m 4][s 2][term 3][lane 64]
//   W3A [s 2][term 3][lane 64]   (5 outputs padded to 16), N = 1 only
//   W3A [s 2][lane 64]           N >= 2: the 16 output rows of the instruction carry the three
//                                 terms of the 5 outputs (l3_row_* below), so ONE A operand meets
//                                 the three activation terms in three instructions per K slice
//   bias b1*pre [64], b2*pre [64], b3 [16] fp32 (N >= 2: b3 in the h-term row of each output)
//
// bf16 variant (BF): one term per weight, rounded to bf16 (nearest even), nothing pre-scaled:
//   W1A [m 4][lane 64]  (K positions 16..31 are zero), W2A [m 4][s 2][lane 64], W3A [s 2][lane 64]
//   (5 outputs padded to 16), bias b1 [64], b2 [64], b3 [16] fp32
template <bool BF>
struct PkT {
  static constexpr size_t OFF_W1A = 0;
  static constexpr size_t W1A_BYTES = BF ? 4 * 64 * 16 : 4 * 2 * 64 * 16;
  static constexpr size_t OFF_W2A = OFF_W1A + W1A_BYTES;
  static constexpr size_t W2A_BYTES = BF ? 4 * 2 * 64 * 16 : 4 * 2 * 3 * 64 * 16;
  static constexpr size_t OFF_W3A = OFF_W2A + W2A_BYTES;
  static constexpr size_t W3A_BYTES = BF ? 2 * 64 * 16 : 2 * 3 * 64 * 16;
  static constexpr size_t OFF_BIAS = OFF_W3A + W3A_BYTES;
  static constexpr size_t BIAS_BYTES = (2 * kH + 16) * 4;
  static constexpr size_t RUN_BYTES = OFF_BIAS + BIAS_BYTES;
  static constexpr size_t LDS_BYTES = OFF_W3A;   // W1A + W2A live in LDS, W3A in registers
};
using Pk = PkT<false>;
using PkB = PkT<true>;

// Layer 3 with the weight terms along the output rows (N >= 2; the logits of a row then need 7
// floats of scratch in its observation row, which has 4N + 2 rewritten columns).  Accumulator
// lane group g holds rows 4g..4g+3: rows 4g + {0,1,2} = terms h, m, l of output g, so their sum
// is lane-local; rows 4g + 3 (g < 3) = term g of output 4, summed by the reader.
template <int N>
struct L3 {
  static constexpr bool kRowTerms = 4 * N + 2 >= 7;
};
__host__ __device__ constexpr int l3_row_output(int i) { return i % 4 < 3 ? i / 4 : (i / 4 < 3 ? 4 : -1); }
__host__ __device__ constexpr int l3_row_term(int i) { return i % 4 < 3 ? i % 4 : i / 4; }

// hidden unit of K position (slice s, lane group gq, element e) in layers 2/3
__host__ __device__ constexpr int hidden_k(int s, int gq, int e) { return 32 * s + 16 * (e / 4) + 4 * gq + (e % 4); }

// One thread per packed bf16 element (all three terms of one weight) or bias value.
template <int N>
__global__ void pack_split_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                  const float* __restrict__ b1, const float* __restrict__ W2,
                                  const float* __restrict__ b2, const float* __restrict__ W3,
                                  const float* __restrict__ b3, int nout) {
  // nout = outputs of the last layer: 5 (policy logits) or 1 (critic value); W3 is [H][nout]
  constexpr int D = 6 * N, KIN = 4 * N + 2;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * Pk::RUN_BYTES;
  W1 += size_t(run) * D * kH;
  b1 += size_t(run) * kH;
  W2 += size_t(run) * kH * kH;
  b2 += size_t(run) * kH;
  W3 += size_t(run) * kH * nout;
  b3 += size_t(run) * nout;
  constexpr int n1 = 4 * 64 * 8, n2 = 4 * 2 * 64 * 8, n3 = 2 * 64 * 8, nb = 2 * kH + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  auto put3 = [&](size_t off, int blk, int lanes, int lane, int e, float v) {
    // blk = index of the [term][lane] group; terms are `lanes` * 16 bytes apart
    uint32_t h, m, l;
    split3(v, h, m, l);
    uint16_t* base = reinterpret_cast<uint16_t*>(out + off) + size_t(blk) * 3 * lanes * 8 + lane * 8 + e;
    base[0] = uint16_t(h >> 16);
    base[size_t(lanes) * 8] = uint16_t(m >> 16);
    base[size_t(2) * lanes * 8] = uint16_t(l >> 16);
  };
  if (idx < n1) {
    const int e = idx % 8, lane = (idx / 8) % 64, m = idx / 512;
    const int gq = lane / 16, k = 8 * (gq & 1) + e, o = 16 * m + lane % 16;
    uint32_t h, mm, l;
    split3(k < KIN ? kPre * W1[size_t(k) * kH + o] : 0.0f, h, mm, l);
    uint16_t* base = reinterpret_cast<uint16_t*>(out + Pk::OFF_W1A) + size_t(m) * 2 * 64 * 8 + lane * 8 + e;
    base[0] = uint16_t((gq < 2 ? h : mm) >> 16);        // combo 0 = (h | m)
    base[64 * 8] = uint16_t((gq < 2 ? h : l) >> 16);    // combo 1 = (h | l)
    return;
  }
  idx -= n1;
  if (idx < n2) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % 2, m = idx / 1024;
    const int k = hidden_k(s, lane / 16, e), o = 16 * m + lane % 16;
    put3(Pk::OFF_W2A, m * 2 + s, 64, lane, e, kPre * W2[size_t(k) * kH + o]);
    return;
  }
  idx -= n2;
  if (idx < n3) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = idx / 512;
    const int k = hidden_k(s, lane / 16, e), o = lane % 16;
    if constexpr (L3<N>::kRowTerms) {
      const int out_o = l3_row_output(o), term = l3_row_term(o);
      uint32_t t3[3] = {0u, 0u, 0u};
      if (out_o >= 0 && out_o < nout) split3(W3[size_t(k) * nout + out_o], t3[0], t3[1], t3[2]);
      reinterpret_cast<uint16_t*>(out + Pk::OFF_W3A)[(size_t(s) * 64 + lane) * 8 + e] = uint16_t(t3[term] >> 16);
    } else {
      put3(Pk::OFF_W3A, s, 64, lane, e, o < nout ? W3[size_t(k) * nout + o] : 0.0f);
    }
    return;
  }
  idx -= n3;
  if (idx < nb) {
    float v;
    if (idx < kH) v = kPre * b1[idx];
    else if (idx < 2 * kH) v = kPre * b2[idx - kH];
    else if constexpr (L3<N>::kRowTerms) {
      const int i = idx - 2 * kH;
      v = (l3_row_output(i) >= 0 && l3_row_output(i) < nout && l3_row_term(i) == 0) ? b3[l3_row_output(i)] : 0.0f;
    } else v = (idx - 2 * kH) < nout ? b3[idx - 2 * kH] : 0.0f;
    reinterpret_cast<float*>(out + Pk::OFF_BIAS)[idx] = v;
  }
}

// ------------------------------------------------------------------------------ operands
struct Terms {   // the three bf16x8 terms of one B (or A) operand
  bf16x8 h, m, l;
};

// Split 8 fp32 activations into the three packed terms.
__device__ __forceinline__ Terms split_operand(const float (&v)[8]) {
  uint32_t h[8], m[8], l[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) split3(v[e], h[e], m[e], l[e]);
  u32x4 ph, pm, pl;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    ph[q] = pack_hi16(h[2 * q], h[2 * q + 1]);
    pm[q] = pack_hi16(m[2 * q], m[2 * q + 1]);
    pl[q] = pack_hi16(l[2 * q], l[2 * q + 1]);
  }
  Terms t;
  t.h = __builtin_bit_cast(bf16x8, ph);
  t.m = __builtin_bit_cast(bf16x8, pm);
  t.l = __builtin_bit_cast(bf16x8, pl);
  return t;
}

#define MPE_MFMA_BF(A, B, C) __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, C, 0, 0, 0)

// acc += A * B from the six significant cross terms, smallest first.
__device__ __forceinline__ f32x4 mma_split(const Terms& a, const Terms& b, f32x4 acc) {
  acc = MPE_MFMA_BF(a.l, b.h, acc);
  acc = MPE_MFMA_BF(a.h, b.l, acc);
  acc = MPE_MFMA_BF(a.m, b.m, acc);
  acc = MPE_MFMA_BF(a.m, b.h, acc);
  acc = MPE_MFMA_BF(a.h, b.m, acc);
  acc = MPE_MFMA_BF(a.h, b.h, acc);
  return acc;
}

// tanh of a pre-activation that arrives already multiplied by 2*log2(e).
__device__ __forceinline__ float tanh_prescaled(float y) {
  return fmaf(-2.0f, hw_rcp(hw_exp2(y) + 1.0f), 1.0f);
}

struct W3Terms {
  Terms s[2];
};

// tanh of 8 accumulator values (tiles 2s and 2s+1 of one batch tile) and their split: the B
// operand of K slice s of the next layer (element e <-> tile 2s + e/4, register e%4).
__device__ __forceinline__ Terms tanh_split(const f32x4& a0, const f32x4& a1) {
  float v[8];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[e] = tanh_prescaled(a0[e]);
    v[4 + e] = tanh_prescaled(a1[e]);
  }
  return split_operand(v);
}

// Policy forward of two 16-row tiles X and Y whose observation rows are in LDS (row stride D).
// Logits of row j go to the first cols of that row (they are rewritten by the next observation).
//
// Schedule.  Matrix-core and vector work only overlap when both are in flight at the same time,
// so the stages are cut where the data dependences allow it: a K slice of the next layer needs
// only HALF of the accumulator tiles of this one (slice s <- tiles 2s, 2s+1), so the tanh + split
// of one half runs on the VALU while the matrix cores finish the other half:
//   split(obs) | L1 m01 | L1 m23 + T1 s0 | L2 s0 + T1 s1 | L2 s1 m01 | L2 s1 m23 + T2 s0 |
//   L3 s0 + T2 s1 | L3 s1
// sched_barrier fences keep the compiler from regrouping the stages.
// VALUE: the network has one output (a critic); it goes to valX[j] / valY[j] and the rows are
// left untouched.
template <int N, bool VALUE = false>
__device__ __forceinline__ void policy_pair(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                            const W3Terms& w3, float* __restrict__ rowsX,
                                            float* __restrict__ rowsY, int lane,
                                            float* __restrict__ valX = nullptr, float* __restrict__ valY = nullptr) {
  constexpr int D = 6 * N;
  const int j = lane & 15, gq = lane >> 4;
  {
    // Opaque zero offset: keeps the (loop-invariant) LDS weight reads inside the step loop, where
    // hoisting them would cost ~100 registers and a wavefront of occupancy.  An integer, not a
    // laundered pointer, so the loads stay ds_read instructions.
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + Pk::OFF_W1A);  // [m][combo][lane64]
  const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + Pk::OFF_W2A);  // [m][s][term][lane64]
  // Layer 1, one output tile: the six cross terms in three instructions, smallest first:
  //   (Wh | Wl) x (Xl | Xh) = hl + lh,  (Wh | Wm) x (Xm | Xm) = hm + mm,  (Wh | Wm) x (Xh | Xh) = hh + mh
  auto layer1 = [&](int m, const Terms& b, const bf16x8& b_lh, f32x4 acc) {
    const bf16x8 a_hm = w1[(m * 2 + 0) * 64 + lane];
    const bf16x8 a_hl = w1[(m * 2 + 1) * 64 + lane];
    acc = MPE_MFMA_BF(a_hl, b_lh, acc);
    acc = MPE_MFMA_BF(a_hm, b.m, acc);
    acc = MPE_MFMA_BF(a_hm, b.h, acc);
    return acc;
  };
  auto load_w2 = [&](int m, int s) {
    Terms a;
    a.h = w2[((m * 2 + s) * 3 + 0) * 64 + lane];
    a.m = w2[((m * 2 + s) * 3 + 1) * 64 + lane];
    a.l = w2[((m * 2 + s) * 3 + 2) * 64 + lane];
    return a;
  };
  // Layer 3, one K slice.  Row-term layout: the one A operand against the three activation terms
  // (all nine cross terms, smallest first); otherwise the six significant ones.
  auto layer3 = [&](const Terms& a, const Terms& b, f32x4 acc) {
    if constexpr (L3<N>::kRowTerms) {
      acc = MPE_MFMA_BF(a.h, b.l, acc);
      acc = MPE_MFMA_BF(a.h, b.m, acc);
      acc = MPE_MFMA_BF(a.h, b.h, acc);
      return acc;
    } else {
      return mma_split(a, b, acc);
    }
  };
  // ---- split(obs): 16 inputs (cols 0..15 of the row; cols >= 4N+2 are zeros or meet zero weights);
  // lanes gq and gq + 2 hold the same 8 inputs
  Terms bx, by;
  bf16x8 bx_lh, by_lh;  // (Xl | Xh): l in K positions 0..15, h in 16..31
  {
    float vx[8], vy[8];
    // rows are D*4 bytes apart (a multiple of 8, not of 16): read as float2
    const float2* xs = reinterpret_cast<const float2*>(rowsX + j * D + 8 * (gq & 1));
    const float2* ys = reinterpret_cast<const float2*>(rowsY + j * D + 8 * (gq & 1));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float2 xv = xs[q], yv = ys[q];
      vx[2 * q] = xv.x; vx[2 * q + 1] = xv.y;
      vy[2 * q] = yv.x; vy[2 * q + 1] = yv.y;
    }
    bx = split_operand(vx);
    by = split_operand(vy);
    bx_lh = gq < 2 ? bx.l : bx.h;
    by_lh = gq < 2 ? by.l : by.h;
  }
  f32x4 accX[4], accY[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    accX[m] = *reinterpret_cast<const f32x4*>(bias + 16 * m + 4 * gq);
    accY[m] = accX[m];
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- L1 m01
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    accX[m] = layer1(m, bx, bx_lh, accX[m]);
    accY[m] = layer1(m, by, by_lh, accY[m]);
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- L1 m23 + T1 s0
  Terms cx0, cy0, cx1, cy1;  // B operands of the next layer, K slices 0 and 1
#pragma unroll
  for (int m = 2; m < 4; ++m) {
    accX[m] = layer1(m, bx, bx_lh, accX[m]);
    accY[m] = layer1(m, by, by_lh, accY[m]);
  }
  cx0 = tanh_split(accX[0], accX[1]);
  cy0 = tanh_split(accY[0], accY[1]);
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    accX[m] = *reinterpret_cast<const f32x4*>(bias + kH + 16 * m + 4 * gq);
    accY[m] = accX[m];
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- L2 s0 (tiles m01 first: their accumulators are free) + T1 s1
  {
    f32x4 tX[2], tY[2];  // L2 accumulators of tiles 2,3 start here; accX/Y[2,3] still hold L1 results
#pragma unroll
    for (int m = 2; m < 4; ++m) {
      tX[m - 2] = *reinterpret_cast<const f32x4*>(bias + kH + 16 * m + 4 * gq);
      tY[m - 2] = tX[m - 2];
    }
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const Terms a = load_w2(m, 0);
      accX[m] = mma_split(a, cx0, accX[m]);
      accY[m] = mma_split(a, cy0, accY[m]);
    }
#pragma unroll
    for (int m = 2; m < 4; ++m) {
      const Terms a = load_w2(m, 0);
      tX[m - 2] = mma_split(a, cx0, tX[m - 2]);
      tY[m - 2] = mma_split(a, cy0, tY[m - 2]);
    }
    cx1 = tanh_split(accX[2], accX[3]);
    cy1 = tanh_split(accY[2], accY[3]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 2; m < 4; ++m) {
      accX[m] = tX[m - 2];
      accY[m] = tY[m - 2];
    }
  }
  // ---- L2 s1 m01
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    const Terms a = load_w2(m, 1);
    accX[m] = mma_split(a, cx1, accX[m]);
    accY[m] = mma_split(a, cy1, accY[m]);
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- L2 s1 m23 + T2 s0
#pragma unroll
  for (int m = 2; m < 4; ++m) {
    const Terms a = load_w2(m, 1);
    accX[m] = mma_split(a, cx1, accX[m]);
    accY[m] = mma_split(a, cy1, accY[m]);
  }
  cx0 = tanh_split(accX[0], accX[1]);
  cy0 = tanh_split(accY[0], accY[1]);
  __builtin_amdgcn_sched_barrier(0);
  // ---- L3 s0 + T2 s1 (5 outputs padded to one 16-wide tile)
  f32x4 zX = *reinterpret_cast<const f32x4*>(bias + 2 * kH + 4 * gq);
  f32x4 zY = zX;
  zX = layer3(w3.s[0], cx0, zX);
  zY = layer3(w3.s[0], cy0, zY);
  cx1 = tanh_split(accX[2], accX[3]);
  cy1 = tanh_split(accY[2], accY[3]);
  __builtin_amdgcn_sched_barrier(0);
  // ---- L3 s1
  zX = layer3(w3.s[1], cx1, zX);
  zY = layer3(w3.s[1], cy1, zY);
  if constexpr (VALUE) {
    // output 0: lane group 0; row-term layout: its three term rows, otherwise register 0
    if (gq == 0) {
      valX[j] = L3<N>::kRowTerms ? (zX[0] + zX[1]) + zX[2] : zX[0];
      valY[j] = L3<N>::kRowTerms ? (zY[0] + zY[1]) + zY[2] : zY[0];
    }
  } else if constexpr (L3<N>::kRowTerms) {
    // lane (j, gq): output gq = sum of its three term rows -> col gq; term gq of output 4 -> col 4 + gq
    rowsX[j * D + gq] = (zX[0] + zX[1]) + zX[2];
    rowsY[j * D + gq] = (zY[0] + zY[1]) + zY[2];
    if (gq < 3) {
      rowsX[j * D + 4 + gq] = zX[3];
      rowsY[j * D + 4 + gq] = zY[3];
    }
  } else {
    // lane (j, gq) holds outputs 4gq + r of row j: outputs 0..3 in group 0, output 4 in group 1
    if (gq == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        rowsX[j * D + r] = zX[r];
        rowsY[j * D + r] = zY[r];
      }
    } else if (gq == 1) {
      rowsX[j * D + 4] = zX[0];
      rowsY[j * D + 4] = zY[0];
    }
  }
}

// LDS plan (bytes).
// ------------------------------------------------------------------------------ bf16 variant
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// One thread per packed bf16 weight or bias value of one run; nout as in pack_split_kernel.
template <int N>
__global__ void pack_bf16_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                 const float* __restrict__ b1, const float* __restrict__ W2,
                                 const float* __restrict__ b2, const float* __restrict__ W3,
                                 const float* __restrict__ b3, int nout) {
  constexpr int D = 6 * N, KIN = 4 * N + 2;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * PkB::RUN_BYTES;
  W1 += size_t(run) * D * kH;
  b1 += size_t(run) * kH;
  W2 += size_t(run) * kH * kH;
  b2 += size_t(run) * kH;
  W3 += size_t(run) * kH * nout;
  b3 += size_t(run) * nout;
  constexpr int n1 = 4 * 64 * 8, n2 = 4 * 2 * 64 * 8, n3 = 2 * 64 * 8, nb = 2 * kH + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n1) {   // [m][lane][e]; k = 8 gq + e for gq < 2, zero above
    const int e = idx % 8, lane = (idx / 8) % 64, m = idx / 512;
    const int gq = lane / 16, k = 8 * gq + e, o = 16 * m + lane % 16;
    reinterpret_cast<uint16_t*>(out + PkB::OFF_W1A)[idx] = f32_to_bf16_rne((gq < 2 && k < KIN) ? W1[size_t(k) * kH + o] : 0.0f);
    return;
  }
  idx -= n1;
  if (idx < n2) {   // [m][s][lane][e]
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % 2, m = idx / 1024;
    reinterpret_cast<uint16_t*>(out + PkB::OFF_W2A)[idx] = f32_to_bf16_rne(W2[size_t(hidden_k(s, lane / 16, e)) * kH + 16 * m + lane % 16]);
    return;
  }
  idx -= n2;
  if (idx < n3) {   // [s][lane][e]
    const int e = idx % 8, lane = (idx / 8) % 64, s = idx / 512, o = lane % 16;
    reinterpret_cast<uint16_t*>(out + PkB::OFF_W3A)[idx] = f32_to_bf16_rne(o < nout ? W3[size_t(hidden_k(s, lane / 16, e)) * nout + o] : 0.0f);
    return;
  }
  idx -= n3;
  if (idx < nb) {
    float v;
    if (idx < kH) v = b1[idx];
    else if (idx < 2 * kH) v = b2[idx - kH];
    else v = (idx - 2 * kH) < nout ? b3[idx - 2 * kH] : 0.0f;
    reinterpret_cast<float*>(out + PkB::OFF_BIAS)[idx] = v;
  }
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Round two floats to bf16 (nearest even) and pack them: low half <- a.
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// tanh of 8 accumulator values (hidden tiles 2s, 2s+1 of one batch tile) rounded to bf16: the B
// operand of K slice s of the next layer.
__device__ __forceinline__ bf16x8 tanh_pack_bf(const f32x4& a0, const f32x4& a1) {
  u32x4 p;
  p[0] = pack_bf16_rne(fast_tanh(a0[0]), fast_tanh(a0[1]));
  p[1] = pack_bf16_rne(fast_tanh(a0[2]), fast_tanh(a0[3]));
  p[2] = pack_bf16_rne(fast_tanh(a1[0]), fast_tanh(a1[1]));
  p[3] = pack_bf16_rne(fast_tanh(a1[2]), fast_tanh(a1[3]));
  return __builtin_bit_cast(bf16x8, p);
}

// bf16 policy forward of two 16-row tiles X and Y (same interface as policy_pair): weights and
// layer inputs bf16, fp32 accumulation and tanh.  Logits of row j go to cols 0..4 of that row.
template <int N, bool VALUE = false>
__device__ __forceinline__ void policy_pair_bf(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                               const W3Terms& w3, float* __restrict__ rowsX,
                                               float* __restrict__ rowsY, int lane,
                                               float* __restrict__ valX = nullptr, float* __restrict__ valY = nullptr) {
  constexpr int D = 6 * N;
  const int j = lane & 15, gq = lane >> 4;
  {
    uint32_t zero = 0;   // see policy_pair: keeps the LDS weight reads inside the step loop
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + PkB::OFF_W1A);  // [m][lane]
  const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + PkB::OFF_W2A);  // [m][s][lane]
  // layer-1 B operands: inputs 8 (gq & 1) .. + 7 of the row; lane groups 2, 3 meet zero weights
  bf16x8 bx, by;
  {
    const float2* xs = reinterpret_cast<const float2*>(rowsX + j * D + 8 * (gq & 1));
    const float2* ys = reinterpret_cast<const float2*>(rowsY + j * D + 8 * (gq & 1));
    u32x4 px, py;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float2 xv = xs[q], yv = ys[q];
      px[q] = pack_bf16_rne(xv.x, xv.y);
      py[q] = pack_bf16_rne(yv.x, yv.y);
    }
    bx = __builtin_bit_cast(bf16x8, px);
    by = __builtin_bit_cast(bf16x8, py);
  }
  f32x4 accX[4], accY[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    accX[m] = *reinterpret_cast<const f32x4*>(bias + 16 * m + 4 * gq);
    accY[m] = accX[m];
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const bf16x8 a = w1[m * 64 + lane];
    accX[m] = MPE_MFMA_BF(a, bx, accX[m]);
    accY[m] = MPE_MFMA_BF(a, by, accY[m]);
  }
  bf16x8 hx[2], hy[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    hx[s] = tanh_pack_bf(accX[2 * s], accX[2 * s + 1]);
    hy[s] = tanh_pack_bf(accY[2 * s], accY[2 * s + 1]);
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    accX[m] = *reinterpret_cast<const f32x4*>(bias + kH + 16 * m + 4 * gq);
    accY[m] = accX[m];
  }
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const bf16x8 a = w2[(m * 2 + s) * 64 + lane];
      accX[m] = MPE_MFMA_BF(a, hx[s], accX[m]);
      accY[m] = MPE_MFMA_BF(a, hy[s], accY[m]);
    }
  }
  f32x4 zX = *reinterpret_cast<const f32x4*>(bias + 2 * kH + 4 * gq);
  f32x4 zY = zX;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    zX = MPE_MFMA_BF(w3.s[s].h, tanh_pack_bf(accX[2 * s], accX[2 * s + 1]), zX);
    zY = MPE_MFMA_BF(w3.s[s].h, tanh_pack_bf(accY[2 * s], accY[2 * s + 1]), zY);
  }
  // lane (j, gq) holds outputs 4gq + r of row j: outputs 0..3 in group 0, output 4 in group 1
  if constexpr (VALUE) {
    if (gq == 0) {
      valX[j] = zX[0];
      valY[j] = zY[0];
    }
  } else {
    if (gq == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        rowsX[j * D + r] = zX[r];
        rowsY[j * D + r] = zY[r];
      }
    } else if (gq == 1) {
      rowsX[j * D + 4] = zX[0];
      rowsY[j * D + 4] = zY[0];
    }
  }
}

// Plain rollout: W1A + W2A and the biases of the policy (its W3A lives in registers).
// Actor-critic rollout (AC): the whole packed image of the policy and of the critic (W1A, W2A,
// W3A, biases each), a value per row, and one arrival counter per 64-env sync group.
template <int N, int EB, bool AC = false, bool BF = false>
struct SmemF32 {
  using P = PkT<BF>;
  static constexpr int D = 6 * N;
  static constexpr int ROWS = EB * N;
  static constexpr size_t OFF_BIAS = AC ? P::OFF_BIAS : P::LDS_BYTES;
  static constexpr size_t OFF_CRITIC = OFF_BIAS + P::BIAS_BYTES;     // AC: the critic's packed image
  static constexpr size_t OFF_OBS = OFF_CRITIC + (AC ? P::RUN_BYTES : 0);
  static constexpr size_t OBS = size_t(ROWS) * D * 4 + 64;           // + zeroed tail: layer 1 reads 16 cols
  static constexpr size_t OFF_NEWPOS = OFF_OBS + OBS;                // [2][ROWS] float2, by step parity
  static constexpr size_t OFF_VALUE = OFF_NEWPOS + size_t(2) * ROWS * 8;   // AC: [ROWS] float
  static constexpr size_t OFF_ARRIVED = OFF_VALUE + (AC ? size_t(ROWS) * 4 : 0);
  static constexpr size_t TOTAL = OFF_ARRIVED + (EB > 64 ? 16 : 0);
  static_assert(OFF_OBS % 16 == 0 && OFF_NEWPOS % 16 == 0 && OFF_CRITIC % 16 == 0 && EB / 64 <= 4, "alignment");
};

// Barrier among the wavefronts of one 64-env sync group inside a larger block.  `arrived` counts
// arrivals since the start of the kernel; `target` = (wavefronts per group) * (barriers so far).
// Every wavefront of the block runs the same number of steps and none leaves early, and a block
// is resident as a whole, so each wait ends.
__device__ __forceinline__ void group_barrier(uint32_t* arrived, uint32_t target, int lane) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  if (lane == 0) __hip_atomic_fetch_add(arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  while (__hip_atomic_load(arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
    __builtin_amdgcn_s_sleep(1);
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// PER_AGENT: rew_traj is [T][TE][N], the mixed per-agent reward; every lane stores its agent's.
// AC (actor-critic outputs): a second network of the same shape with one output, `packed_critic`,
// is evaluated on every observation acted on, and the log-probability of the sampled action is
// recorded (paper Sec. 3.2: IPPO / MAPPO; App. G: two tanh layers of width 64).  A block is then
// EB / 64 independent 64-env sync groups that share the two staged networks.
template <int N, int EB, int MINW, bool PER_AGENT, bool AC, bool BF>
__global__ __launch_bounds__(EB * N, MINW) void rollout_policy_f32_kernel(RolloutArgs A, const uint8_t* __restrict__ packed,
                                                                          const uint8_t* __restrict__ packed_critic,
                                                                          int per_run_weights, uint32_t groups,
                                                                          uint32_t groups_per_xcd) {
  using M = SmemF32<N, EB, AC, BF>;
  using P = PkT<BF>;

  constexpr int D = 6 * N, ROWS = EB * N, THREADS = ROWS;
  static_assert(THREADS % 64 == 0, "block must be whole wavefronts");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* wsm = smem;
  float* bias = reinterpret_cast<float*>(smem + M::OFF_BIAS);
  float* tile = reinterpret_cast<float*>(smem + M::OFF_OBS);
  float2* newpos = reinterpret_cast<float2*>(smem + M::OFF_NEWPOS);
  const uint8_t* csm = smem + M::OFF_CRITIC;                                         // AC only
  const float* cbias = reinterpret_cast<const float*>(smem + M::OFF_CRITIC + P::OFF_BIAS);
  float* values = reinterpret_cast<float*>(smem + M::OFF_VALUE);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int el = tid / N, i = tid - el * N;          // env within block, agent
  const size_t TE = A.TE;
  // XCD-aware mapping: the hardware deals block b to XCD b % 8; giving each XCD one contiguous
  // range of env groups lets the partial cache lines that neighbouring groups write per step
  // (actions 3*EB bytes, done EB bytes) merge in one L2 instead of being written back apart.
  const uint32_t grp = (blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3);
  if (grp >= groups) return;  // whole block, before any barrier
  const size_t g0 = size_t(grp) * EB;
  const size_t g = g0 + el;
  const bool valid = g < TE;
  const uint32_t gc = valid ? uint32_t(g) : uint32_t(g0);
  const uint32_t run = gc / A.E;
  const uint32_t env = gc - run * A.E;
  const size_t left = TE - g0;
  const int nvalid = left < size_t(EB) ? int(left) : EB;   // valid envs in this block
  // rows of this wavefront that belong to valid envs
  const int wave_rows = min(max(nvalid * N - wave * 64, 0), 64);

  // ---- stage this block's weights (the run of its first env): W1A, W2A, biases in LDS; W3A in registers
  const uint8_t* run_weights = packed + (per_run_weights ? size_t(uint32_t(g0) / A.E) * P::RUN_BYTES : 0);
  // A operands of layer 3 from a packed image (global memory or LDS)
  auto load_w3 = [&](const uint8_t* image) {
    W3Terms w;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if constexpr (BF || L3<N>::kRowTerms) {
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
    if constexpr (AC) {
      for (int k = tid; k < int(P::RUN_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* csrc = reinterpret_cast<const uint4*>(
          packed_critic + (per_run_weights ? size_t(uint32_t(g0) / A.E) * P::RUN_BYTES : 0));
      uint4* cdst = reinterpret_cast<uint4*>(smem + M::OFF_CRITIC);
      for (int k = tid; k < int(P::RUN_BYTES / 16); k += THREADS) cdst[k] = csrc[k];
    } else {
      for (int k = tid; k < int(P::LDS_BYTES / 16); k += THREADS) dst[k] = src[k];
      const uint4* bsrc = reinterpret_cast<const uint4*>(run_weights + P::OFF_BIAS);
      uint4* bdst = reinterpret_cast<uint4*>(bias);
      for (int k = tid; k < int(P::BIAS_BYTES / 16); k += THREADS) bdst[k] = bsrc[k];
    }
    if (tid < 16) tile[ROWS * D + tid] = 0.0f;
    if constexpr (EB > 64) {
      if (tid < EB / 64) reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED)[tid] = 0u;
    }
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
  __syncthreads();  // weights, biases, zero tail staged; from here on wavefronts only meet at (C)

  // Output addresses = uniform per-step base (advanced once per step, lives in SGPRs) + a
  // 32-bit lane offset that never changes.
  const size_t wave_row0 = (g0 * N + size_t(wave) * 64) * D;   // float offset of this wavefront's rows in a slice
  float* obs_p = A.obs_traj ? A.obs_traj + wave_row0 : nullptr;
  uint8_t* act_base = A.act_traj;
  float* rew_base = A.rew_traj;
  uint8_t* done_base = A.done_traj;
  float* logp_base = A.logp_traj;
  float* value_base = A.value_traj;
  const uint32_t row_off = uint32_t(gc) * N + i;      // index of this agent inside a time slice
  const bool env_writer = valid && i == 0;            // the lane that stores per-env outputs
  uint32_t step = A.abs_step;
  const float* wtile = tile + wave * (64 * D);        // this wavefront's rows
  uint32_t* arrived = reinterpret_cast<uint32_t*>(smem + M::OFF_ARRIVED) + wave / N;   // EB > 64 only

  // Critic forward of this wavefront's rows: values[row] (wave-local rows).
  auto critic_rows = [&]() {
#pragma unroll 1
    for (int pr = 0; pr < 2; ++pr) {
      float* rows = tile + (wave * 64 + pr * 32) * D;
      float* vals = values + wave * 64 + pr * 32;
      const W3Terms wc = load_w3(csm);
      if constexpr (BF) policy_pair_bf<N, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
      else policy_pair<N, true>(csm, cbias, wc, rows, rows + 16 * D, lane, vals, vals + 16);
    }
  };

  // Stream this wavefront's rows of the tile to dst (its slot in a [env][N][D] slice).
  auto flush_rows = [&](float* dst) {
    const bool vec4 = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
    if (vec4 && wave_rows == 64) stream_out_full<64 * D / 4>(wtile, dst, lane);
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
    for (int pr = 0; pr < 2; ++pr) {
      float* rows = tile + (wave * 64 + pr * 32) * D;
      if constexpr (AC) w3 = load_w3(wsm);
      if constexpr (BF) policy_pair_bf<N>(wsm, bias, w3, rows, rows + 16 * D, lane);
      else policy_pair<N>(wsm, bias, w3, rows, rows + 16 * D, lane);
    }
    wave_sync();
    float z[kNumActions];
#pragma unroll
    for (int k = 0; k < kNumActions; ++k) z[k] = tile[tid * D + k];
    if constexpr (!BF && L3<N>::kRowTerms) z[4] = (z[4] + tile[tid * D + 5]) + tile[tid * D + 6];
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
    float2* np = newpos + (t & 1) * ROWS;
    np[tid] = make_float2(px, py);
    // (C) new positions of every agent of every env of this 64-env group are visible
    if constexpr (EB == 64) __syncthreads();
    else if constexpr (N > 1) group_barrier(arrived, uint32_t(N) * uint32_t(t + 1), lane);
    else wave_sync();

#pragma unroll
    for (int a = 0; a < N; ++a) {
      const float2 p = np[el * N + a];
      qx[a] = p.x;
      qy[a] = p.y;
    }
    // shared coverage reward, evaluated by every lane (N*N distances), stored by agent 0
    {
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
      if constexpr (PER_AGENT) {
        uint32_t overlaps = 0;
#pragma unroll
        for (int a = 0; a < N; ++a) {
          if (a != i) {
            const float dx = px - qx[a], dy = py - qy[a];
            overlaps += fmaf(dx, dx, dy * dy) < A.ph.two_r_sq ? 1u : 0u;
          }
        }
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

template <int N, int EB, int MINW, bool PER_AGENT, bool AC, bool BF>
hipError_t rollout_impl(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const void* critic = nullptr) {
  using M = SmemF32<N, EB, AC, BF>;
  auto kern = rollout_policy_f32_kernel<N, EB, MINW, PER_AGENT, AC, BF>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(M::TOTAL));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const uint32_t groups = (A.TE + EB - 1) / EB;
  const uint32_t per_xcd = (groups + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(EB * N), M::TOTAL, s, A, static_cast<const uint8_t*>(pb.packed),
                     static_cast<const uint8_t*>(critic), int(A.TE != A.E), groups, per_xcd);
  return hipGetLastError();
}

template <int N>
hipError_t pack_impl(PolicyBuffers& pb, int R, const float* W1, const float* b1, const float* W2,
                     const float* b2, const float* W3, const float* b3, int nout, bool bf16, hipStream_t s) {
  const size_t run_bytes = bf16 ? PkB::RUN_BYTES : Pk::RUN_BYTES;
  if (hipError_t e = ensure_policy_bytes(pb, size_t(R) * run_bytes); e != hipSuccess) return e;
  constexpr int total = 4 * 64 * 8 + 4 * 2 * 64 * 8 + 2 * 64 * 8 + 2 * kH + 16;   // threads: one per weight / bias
  dim3 grid((total + 255) / 256, R);
  if (bf16)
    hipLaunchKernelGGL(pack_bf16_kernel<N>, grid, dim3(256), 0, s, static_cast<uint8_t*>(pb.packed), W1, b1, W2,
                       b2, W3, b3, nout);
  else
    hipLaunchKernelGGL(pack_split_kernel<N>, grid, dim3(256), 0, s, static_cast<uint8_t*>(pb.packed), W1, b1, W2,
                       b2, W3, b3, nout);
  return hipGetLastError();
}

// Compute units of the current device (queried once per process).
uint32_t compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return uint32_t(cus);
}

// Envs per block.  64 (N wavefronts, one block barrier per step) is the general shape: three
// blocks are resident per CU, and with several runs every block must lie inside one run.  When
// one run has at least one 256-env block per CU, blocks of 256 envs = four independent 64-env
// sync groups (12 wavefronts, per-group arrival counters) fill the chip in whole rounds with no
// tail of single resident blocks: measured 2.31 ms against 2.37 ms at 65,536 envs x 3 agents.
// (Two 128-env blocks per CU with ONE block barrier among six wavefronts were slower: 2.97 ms.)
template <int N, bool BF>
hipError_t launch_n(const RolloutArgs& A, const PolicyBuffers& pb, hipStream_t s, const char** why) {
  const bool one_run = A.TE == A.E;
  const bool per_agent = A.ph.reward_mode == 1;
  if (one_run && A.TE / 256 >= compute_units())
    return per_agent ? rollout_impl<N, 256, 3, true, false, BF>(A, pb, s) : rollout_impl<N, 256, 3, false, false, BF>(A, pb, s);
  if (one_run || A.E % 64 == 0)
    return per_agent ? rollout_impl<N, 64, 3, true, false, BF>(A, pb, s) : rollout_impl<N, 64, 3, false, false, BF>(A, pb, s);
  *why = "with several runs, num_envs per run must be a multiple of 64";
  return hipSuccess;
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
  if (one_run ? A.TE / 256 >= compute_units() / 2 : A.E % 256 == 0)
    return per_agent ? rollout_impl<N, 256, 3, true, true, BF>(A, pb, s, critic.packed)
                     : rollout_impl<N, 256, 3, false, true, BF>(A, pb, s, critic.packed);
  if (one_run || A.E % 64 == 0)
    return per_agent ? rollout_impl<N, 64, 3, true, true, BF>(A, pb, s, critic.packed)
                     : rollout_impl<N, 64, 3, false, true, BF>(A, pb, s, critic.packed);
  *why = "with several runs, num_envs per run must be a multiple of 64";
  return hipSuccess;
}

}  // namespace

bool f32_supported(int N, int H) { return H == kH && N >= 1 && N <= 3; }

hipError_t pack_policy_f32(PolicyBuffers& pb, int N, int R, const float* W1, const float* b1, const float* W2,
                           const float* b2, const float* W3, const float* b3, int nout, bool bf16, hipStream_t s) {
  switch (N) {
    case 1: return pack_impl<1>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    case 2: return pack_impl<2>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    case 3: return pack_impl<3>(pb, R, W1, b1, W2, b2, W3, b3, nout, bf16, s);
    default: return hipErrorInvalidValue;
  }
}

#define MPE_BY_N_AND_DTYPE(FN, ...)                                              \
  switch (N) {                                                                   \
    case 1: return bf16 ? FN<1, true>(__VA_ARGS__) : FN<1, false>(__VA_ARGS__);  \
    case 2: return bf16 ? FN<2, true>(__VA_ARGS__) : FN<2, false>(__VA_ARGS__);  \
    case 3: return bf16 ? FN<3, true>(__VA_ARGS__) : FN<3, false>(__VA_ARGS__);  \
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
