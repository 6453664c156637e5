// The 64-wide two-layer tanh MLP of the fused rollout kernels on the 16-bit matrix cores: packing of
// the weights into A-operand order, the operand splits (sums of fp16 terms) that give fp32 products,
// and the forward pass of two 16-row tiles (fp32 split-operand and bf16 variants).  Shared by the kernels
// of both scenarios; everything is templated on a shape S:
//   S::D         floats per observation row in the LDS tile (row stride)
//   S::KIN       leading inputs of a row that the first layer reads (<= 64; the rest of the row is
//                zero in every observation); up to 16 inputs ride in half of an instruction's K
//                positions and the other half carries a second term (S::kWideIn false), 17..32 inputs
//                fill the K slice and layer 1 takes the six instructions of any other product,
//                33..64 inputs are two such slices (S::kSlices1)
//   S::kRowTerms layer 3 with the weight terms along the output rows (needs 7 scratch floats per row)
#pragma once

#include "mpe_policy_common.h"

namespace mpe {

template <int D_, int KIN_>
struct NetShape {
  static constexpr int D = D_;
  static constexpr int KIN = KIN_;
  static constexpr bool kRowTerms = KIN_ >= 7;
  static constexpr bool kWideIn = KIN_ > 16;
  static constexpr int kSlices1 = KIN_ > 32 ? 2 : 1;     // K slices of layer 1
  static_assert(KIN_ <= 64 && KIN_ <= D_ && D_ % 2 == 0, "layer 1 reads at most two K slices, rows are float2-aligned");
};

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kH = 64;                    // hidden width
constexpr float kPre = 2.0f * kLog2e;     // both tanh layers get pre-activations already times 2*log2(e)

// ------------------------------------------------------------------------------ operand splits
// fp32 products on the 16-bit matrix cores: an operand is a sum of fp16 terms, a product the sum of the cross
// terms that matter, accumulated in fp32.
// Three terms, x = h + m + l: h = x truncated to fp16 (11 significant bits), m = (x - h) truncated,
// l = x - h - m truncated; both differences are exact in fp32.  11 + 11 + 2 bits cover the 24 of an fp32
// number, so the split is EXACT for |x| >= 0.5 (and < 65,504); below that the third term lies on fp16's
// subnormal grid and x is represented to within 2^-24 ABSOLUTE.  The matrix instruction takes subnormal
// fp16 inputs at full precision (checked on the chip).  Truncation (round toward zero) keeps every term of
// the sign of x and is one instruction for two values (v_cvt_pkrtz_f16_f32); a difference is one mixed-
// precision fma that reads the fp16 half in place (v_fma_mix_f32): 7 instructions per PAIR of values, and
// the packed pairs are the matrix operands as they are.  (An fp32 = 3 x bf16 split, 8 + 8 + 8 bits, is exact
// everywhere but costs 11 instructions per pair: and, sub, and, sub per value and three byte-permutes.)
// Used for the observations and the weights of layers 1 and 3.
// Two terms, each rounded to NEAREST (split2_pair below): 4 instructions per pair, |x - h - m| <= 2^-23 |x|,
// one unit in the last place of fp32.  Used where the operand already carries an error of that size: the
// hidden activations (outputs of the hardware tanh, ~1e-7 absolute) and the weights of layer 2 (stored
// pre-scaled by 2 log2(e), a product that is itself rounded to fp32).  Measured against the float64
// networks on 6e5 recorded rows, the outputs' mean error is 1.4e-7 with either split (a plain float32
// evaluation with a correctly rounded tanh: 0.7e-7): it is set by the tanh, not by the split.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// c - a, where a is the low (HI = false) or high half of a packed fp16 pair: one v_fma_mix_f32, which
// widens the half in place.  (Written as a * -1 + c in plain C++ the compiler folds it into a conversion
// and a subtraction, two instructions.)
template <bool HI>
__device__ __forceinline__ float sub_half(uint32_t pair, float c) {
  float d;
  if constexpr (HI) asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(c));
  else asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(c));
  return d;
}

// Two values at once: the packed pairs (low half <- x0) of the three terms.
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t& ph, uint32_t& pm, uint32_t& pl) {
  ph = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x0, x1));
  const float r0 = sub_half<false>(ph, x0);
  const float r1 = sub_half<true>(ph, x1);
  pm = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r0, r1));
  const float s0 = sub_half<false>(pm, r0);
  const float s1 = sub_half<true>(pm, r1);
  pl = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(s0, s1));
}
// Two terms, each rounded to nearest: x = h + m + d with |d| <= 2^-23 |x| (h keeps 11 significant bits, the
// remainder is at most half a unit of h's last place and m keeps 11 bits of it), 4 instructions per pair.
__device__ __forceinline__ void split2_pair(float x0, float x1, uint32_t& ph, uint32_t& pm) {
  typedef float f32x2_ __attribute__((ext_vector_type(2)));
  const f32x2_ x = {x0, x1};
  ph = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));       // v_cvt_pk_f16_f32, nearest even
  const f32x2_ r = {sub_half<false>(ph, x0), sub_half<true>(ph, x1)};
  pm = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, f16x2));
}
// One value: the 16-bit patterns of its three terms.
__device__ __forceinline__ void split3(float x, uint32_t& h, uint32_t& m, uint32_t& l) {
  uint32_t ph, pm, pl;
  split3_pair(x, 0.0f, ph, pm, pl);
  h = ph & 0xFFFFu;
  m = pm & 0xFFFFu;
  l = pl & 0xFFFFu;
}

// Packed per-run layout (bytes).  A operands of v_mfma_f32_16x16x32_f16 (fp16 terms of the split): lane (i = lane%16,
// gq = lane/16) holds weights [k = 8 gq + e][out = 16 m + i], e = 0..7 (16 bytes), per term.
//   W1A [m 4][combo 2][lane 64]  layer 1 has only 16 inputs, half of the instruction's K = 32, so
//                                 two cross terms share one instruction: K positions 0..15 (lanes
//                                 gq < 2) carry one term of input k' = 8 (gq & 1) + e, positions
//                                 16..31 (gq >= 2) another term of the same inputs.
//                                 combo 0 = (h | m), combo 1 = (h | l)
//   W1A [m 4][s][term 3][lane 64]  shapes with 17..64 inputs (kWideIn; s = K slice, one or two): k = 32 s + 8 gq + e,
//                                 all three terms
//   W2A [m 4][s 2][term 2][lane 64]  the two-term split (split2_pair) of the pre-scaled weights
//   W3A [s 2][term 3][lane 64]   (5 outputs padded to 16), shapes without kRowTerms only
//   W3A [s 2][lane 64]           kRowTerms: the 16 output rows of the instruction carry the three
//                                 terms of the 5 outputs (l3_row_* below), so ONE A operand meets
//                                 the three activation terms in three instructions per K slice
//   bias b1*pre [64], b2*pre [64], b3 [16] fp32 (kRowTerms: b3 in the h-term row of each output)
//
// bf16 variant (BF): one term per weight, rounded to bf16 (nearest even), nothing pre-scaled:
//   W1A [m 4][s][lane 64]  (K positions 16..31 are zero unless kWideIn; s = K slice as above), W2A [m 4][s 2][lane 64], W3A [s 2][lane 64]
//   (5 outputs padded to 16), bias b1 [64], b2 [64], b3 [16] fp32
template <bool BF, bool WIDE_IN = false, int KS1 = 1>
struct PkT {
  static_assert(KS1 == 1 || WIDE_IN, "two K slices only in the wide-input layout");
  static constexpr size_t OFF_W1A = 0;
  static constexpr size_t W1A_BYTES = BF ? 4 * KS1 * 64 * 16 : (WIDE_IN ? 4 * KS1 * 3 * 64 * 16 : 4 * 2 * 64 * 16);
  static constexpr size_t OFF_W2A = OFF_W1A + W1A_BYTES;
  static constexpr size_t W2A_BYTES = BF ? 4 * 2 * 64 * 16 : 4 * 2 * 2 * 64 * 16;
  static constexpr size_t OFF_W3A = OFF_W2A + W2A_BYTES;
  static constexpr size_t W3A_BYTES = BF ? 2 * 64 * 16 : 2 * 3 * 64 * 16;
  static constexpr size_t OFF_BIAS = OFF_W3A + W3A_BYTES;
  static constexpr size_t BIAS_BYTES = (2 * kH + 16) * 4;
  static constexpr size_t RUN_BYTES = OFF_BIAS + BIAS_BYTES;
  static constexpr size_t LDS_BYTES = OFF_W3A;   // W1A + W2A live in LDS, W3A in registers
};
using Pk = PkT<false>;
using PkB = PkT<true>;

// Layer 3 with the weight terms along the output rows (kRowTerms; the logits of a row then need 7
// floats of scratch in its observation row, which has KIN rewritten columns).  Accumulator
// lane group g holds rows 4g..4g+3: rows 4g + {0,1,2} = terms h, m, l of output g, so their sum
// is lane-local; rows 4g + 3 (g < 3) = term g of output 4, summed by the reader.
__host__ __device__ constexpr int l3_row_output(int i) { return i % 4 < 3 ? i / 4 : (i / 4 < 3 ? 4 : -1); }
__host__ __device__ constexpr int l3_row_term(int i) { return i % 4 < 3 ? i % 4 : i / 4; }

// hidden unit of K position (slice s, lane group gq, element e) in layers 2/3
__host__ __device__ constexpr int hidden_k(int s, int gq, int e) { return 32 * s + 16 * (e / 4) + 4 * gq + (e % 4); }

// Threads of either pack kernel: one per weight (layer 1 padded to its K slices) or bias value.
template <typename S>
constexpr int pack_threads() { return 4 * S::kSlices1 * 64 * 8 + 4 * 2 * 64 * 8 + 2 * 64 * 8 + 2 * kH + 16; }

// One thread per packed bf16 element (all three terms of one weight) or bias value.
template <typename S>
__global__ void pack_split_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                  const float* __restrict__ b1, const float* __restrict__ W2,
                                  const float* __restrict__ b2, const float* __restrict__ W3,
                                  const float* __restrict__ b3, int nout) {
  // nout = outputs of the last layer: 5 (policy logits) or 1 (critic value); W3 is [H][nout]
  using Pk = PkT<false, S::kWideIn, S::kSlices1>;
  constexpr int D = S::D, KIN = S::KIN, KS1 = S::kSlices1;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * Pk::RUN_BYTES;
  W1 += size_t(run) * D * kH;
  b1 += size_t(run) * kH;
  W2 += size_t(run) * kH * kH;
  b2 += size_t(run) * kH;
  W3 += size_t(run) * kH * nout;
  b3 += size_t(run) * nout;
  constexpr int n1 = 4 * KS1 * 64 * 8, n2 = 4 * 2 * 64 * 8, n3 = 2 * 64 * 8, nb = 2 * kH + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  auto put3 = [&](size_t off, int blk, int lanes, int lane, int e, float v) {
    // blk = index of the [term][lane] group; terms are `lanes` * 16 bytes apart
    uint32_t h, m, l;
    split3(v, h, m, l);
    uint16_t* base = reinterpret_cast<uint16_t*>(out + off) + size_t(blk) * 3 * lanes * 8 + lane * 8 + e;
    base[0] = uint16_t(h);
    base[size_t(lanes) * 8] = uint16_t(m);
    base[size_t(2) * lanes * 8] = uint16_t(l);
  };
  if (idx < n1) {
    const int e = idx % 8, lane = (idx / 8) % 64;
    if constexpr (S::kWideIn) {
      const int sl = (idx / 512) % KS1, mw = idx / (512 * KS1);
      const int k = 32 * sl + 8 * (lane / 16) + e;
      put3(Pk::OFF_W1A, mw * KS1 + sl, 64, lane, e, k < KIN ? kPre * W1[size_t(k) * kH + 16 * mw + lane % 16] : 0.0f);
      return;
    }
    const int m = idx / 512;
    const int gq = lane / 16, k = 8 * (gq & 1) + e, o = 16 * m + lane % 16;
    uint32_t h, mm, l;
    split3(k < KIN ? kPre * W1[size_t(k) * kH + o] : 0.0f, h, mm, l);
    uint16_t* base = reinterpret_cast<uint16_t*>(out + Pk::OFF_W1A) + size_t(m) * 2 * 64 * 8 + lane * 8 + e;
    base[0] = uint16_t(gq < 2 ? h : mm);        // combo 0 = (h | m)
    base[64 * 8] = uint16_t(gq < 2 ? h : l);    // combo 1 = (h | l)
    return;
  }
  idx -= n1;
  if (idx < n2) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = (idx / 512) % 2, m = idx / 1024;
    const int k = hidden_k(s, lane / 16, e), o = 16 * m + lane % 16;
    uint32_t ph, pm;
    split2_pair(kPre * W2[size_t(k) * kH + o], 0.0f, ph, pm);
    uint16_t* base = reinterpret_cast<uint16_t*>(out + Pk::OFF_W2A) + size_t(m * 2 + s) * 2 * 64 * 8 + lane * 8 + e;
    base[0] = uint16_t(ph & 0xFFFFu);
    base[64 * 8] = uint16_t(pm & 0xFFFFu);
    return;
  }
  idx -= n2;
  if (idx < n3) {
    const int e = idx % 8, lane = (idx / 8) % 64, s = idx / 512;
    const int k = hidden_k(s, lane / 16, e), o = lane % 16;
    if constexpr (S::kRowTerms) {
      const int out_o = l3_row_output(o), term = l3_row_term(o);
      uint32_t t3[3] = {0u, 0u, 0u};
      if (out_o >= 0 && out_o < nout) split3(W3[size_t(k) * nout + out_o], t3[0], t3[1], t3[2]);
      reinterpret_cast<uint16_t*>(out + Pk::OFF_W3A)[(size_t(s) * 64 + lane) * 8 + e] = uint16_t(t3[term]);
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
    else if constexpr (S::kRowTerms) {
      const int i = idx - 2 * kH;
      v = (l3_row_output(i) >= 0 && l3_row_output(i) < nout && l3_row_term(i) == 0) ? b3[l3_row_output(i)] : 0.0f;
    } else v = (idx - 2 * kH) < nout ? b3[idx - 2 * kH] : 0.0f;
    reinterpret_cast<float*>(out + Pk::OFF_BIAS)[idx] = v;
  }
}

// ------------------------------------------------------------------------------ operands
struct Terms {   // the three terms of one B (or A) operand: 8 x 16 bits each (fp16; one bf16 term in the bf16 variant)
  bf16x8 h, m, l;
};

// Split 8 fp32 activations into the three packed terms.
__device__ __forceinline__ Terms split_operand(const float (&v)[8]) {
  u32x4 ph, pm, pl;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t a, b, c;
    split3_pair(v[2 * q], v[2 * q + 1], a, b, c);
    ph[q] = a;
    pm[q] = b;
    pl[q] = c;
  }
  Terms t;
  t.h = __builtin_bit_cast(bf16x8, ph);
  t.m = __builtin_bit_cast(bf16x8, pm);
  t.l = __builtin_bit_cast(bf16x8, pl);
  return t;
}

// The two-term split of 8 hidden activations (l is left unset and never read).
__device__ __forceinline__ Terms split_activation(const float (&v)[8]) {
  u32x4 ph, pm;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t a, b;
    split2_pair(v[2 * q], v[2 * q + 1], a, b);
    ph[q] = a;
    pm[q] = b;
  }
  Terms t;
  t.h = __builtin_bit_cast(bf16x8, ph);
  t.m = __builtin_bit_cast(bf16x8, pm);
  return t;
}

#define MPE_MFMA_BF(A, B, C) __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, C, 0, 0, 0)
// the same shape on fp16 operands, for the terms of the three-term split (stored as raw 8 x 16 bits)
#define MPE_MFMA_SPLIT(A, B, C) \
  __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, A), __builtin_bit_cast(f16x8, B), C, 0, 0, 0)

// acc += A * B from the six cross terms of weight >= 2^-22 (terms h, m, l weigh 1, 2^-11, 2^-22; the
// dropped m l, l m, l l are below 2^-33 of the product), smallest first.
__device__ __forceinline__ f32x4 mma_split(const Terms& a, const Terms& b, f32x4 acc) {
  acc = MPE_MFMA_SPLIT(a.l, b.h, acc);
  acc = MPE_MFMA_SPLIT(a.h, b.l, acc);
  acc = MPE_MFMA_SPLIT(a.m, b.m, acc);
  acc = MPE_MFMA_SPLIT(a.m, b.h, acc);
  acc = MPE_MFMA_SPLIT(a.h, b.m, acc);
  acc = MPE_MFMA_SPLIT(a.h, b.h, acc);
  return acc;
}

// Two-term operands on both sides (terms h, m of a and b): the four cross terms, smallest first.
__device__ __forceinline__ f32x4 mma_split22(const Terms& a, const Terms& b, f32x4 acc) {
  acc = MPE_MFMA_SPLIT(a.m, b.m, acc);
  acc = MPE_MFMA_SPLIT(a.m, b.h, acc);
  acc = MPE_MFMA_SPLIT(a.h, b.m, acc);
  acc = MPE_MFMA_SPLIT(a.h, b.h, acc);
  return acc;
}

// Three-term weights a against a two-term activation operand b (split_activation): the five cross terms of
// weight >= 2^-23, smallest first.
__device__ __forceinline__ f32x4 mma_split_act(const Terms& a, const Terms& b, f32x4 acc) {
  acc = MPE_MFMA_SPLIT(a.l, b.h, acc);
  return mma_split22(a, b, acc);
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
  return split_activation(v);
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
// The network itself, registers in and out: vx / vy = this lane's 8 inputs of tile X / Y (lane (j, gq):
// inputs 8 (gq & 1) .. + 7 of row j; kWideIn: inputs 8 gq .. + 7, zero beyond the row), zX / zY = the layer-3 accumulators of the two tiles.
template <typename S>
__device__ __forceinline__ void policy_core(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                            const W3Terms& w3, const float (&vx)[S::kSlices1][8],
                                            const float (&vy)[S::kSlices1][8], f32x4& zX, f32x4& zY, int lane) {
  using Pk = PkT<false, S::kWideIn, S::kSlices1>;
  constexpr int KS1 = S::kSlices1;
  const int gq = lane >> 4;
  // The network runs at a raised wavefront priority: a wavefront that has matrix instructions to issue goes
  // ahead of the wavefronts of its SIMD that are in the (vector-only) env step, whose instructions then fill
  // the gaps (measured on the 65,536-env rollout: 2.11-2.15 -> 2.00-2.03 ms on one box, no change on a
  // faster one; priority 3 is the same as 2).
  __builtin_amdgcn_s_setprio(2);
  {
    // Opaque zero offset: keeps the (loop-invariant) LDS weight reads inside the step loop, where
    // hoisting them would cost ~100 registers and a wavefront of occupancy.  An integer, not a
    // laundered pointer, so the loads stay ds_read instructions.
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + Pk::OFF_W1A);  // [m][combo][lane64]; kWideIn: [m][term][lane64]
  const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + Pk::OFF_W2A);  // [m][s][term 2][lane64]
  // Layer 1, one output tile: the six cross terms in three instructions, smallest first:
  //   (Wh | Wl) x (Xl | Xh) = hl + lh,  (Wh | Wm) x (Xm | Xm) = hm + mm,  (Wh | Wm) x (Xh | Xh) = hh + mh
  auto layer1 = [&](int m, const Terms (&b)[KS1], const bf16x8& b_lh, f32x4 acc) {
    if constexpr (S::kWideIn) {   // 17..64 inputs fill one or two K slices: the six cross terms, one instruction each
#pragma unroll
      for (int s = 0; s < KS1; ++s) {
        Terms a;
        a.h = w1[((m * KS1 + s) * 3 + 0) * 64 + lane];
        a.m = w1[((m * KS1 + s) * 3 + 1) * 64 + lane];
        a.l = w1[((m * KS1 + s) * 3 + 2) * 64 + lane];
        acc = mma_split(a, b[s], acc);
      }
      return acc;
    }
    const bf16x8 a_hm = w1[(m * 2 + 0) * 64 + lane];
    const bf16x8 a_hl = w1[(m * 2 + 1) * 64 + lane];
    acc = MPE_MFMA_SPLIT(a_hl, b_lh, acc);
    acc = MPE_MFMA_SPLIT(a_hm, b[0].m, acc);
    acc = MPE_MFMA_SPLIT(a_hm, b[0].h, acc);
    return acc;
  };
  auto load_w2 = [&](int m, int s) {
    Terms a;
    a.h = w2[((m * 2 + s) * 2 + 0) * 64 + lane];
    a.m = w2[((m * 2 + s) * 2 + 1) * 64 + lane];
    return a;
  };
  // Layer 3, one K slice.  Row-term layout: the one A operand against the three activation terms
  // (all nine cross terms, smallest first); otherwise the six significant ones.
  auto layer3 = [&](const Terms& a, const Terms& b, f32x4 acc) {
    if constexpr (S::kRowTerms) {
      acc = MPE_MFMA_SPLIT(a.h, b.m, acc);
      acc = MPE_MFMA_SPLIT(a.h, b.h, acc);
      return acc;
    } else {
      return mma_split_act(a, b, acc);
    }
  };
  // ---- split(obs): 16 inputs (cols 0..15 of the row; cols >= 4N+2 are zeros or meet zero weights);
  // lanes gq and gq + 2 hold the same 8 inputs
  Terms bx[KS1], by[KS1];
  bf16x8 bx_lh, by_lh;  // (Xl | Xh): l in K positions 0..15, h in 16..31 (shapes of up to 16 inputs)
  {
#pragma unroll
    for (int s = 0; s < KS1; ++s) {
      bx[s] = split_operand(vx[s]);
      by[s] = split_operand(vy[s]);
    }
    bx_lh = gq < 2 ? bx[0].l : bx[0].h;
    by_lh = gq < 2 ? by[0].l : by[0].h;
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
      accX[m] = mma_split22(a, cx0, accX[m]);
      accY[m] = mma_split22(a, cy0, accY[m]);
    }
#pragma unroll
    for (int m = 2; m < 4; ++m) {
      const Terms a = load_w2(m, 0);
      tX[m - 2] = mma_split22(a, cx0, tX[m - 2]);
      tY[m - 2] = mma_split22(a, cy0, tY[m - 2]);
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
    accX[m] = mma_split22(a, cx1, accX[m]);
    accY[m] = mma_split22(a, cy1, accY[m]);
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- L2 s1 m23 + T2 s0
#pragma unroll
  for (int m = 2; m < 4; ++m) {
    const Terms a = load_w2(m, 1);
    accX[m] = mma_split22(a, cx1, accX[m]);
    accY[m] = mma_split22(a, cy1, accY[m]);
  }
  cx0 = tanh_split(accX[0], accX[1]);
  cy0 = tanh_split(accY[0], accY[1]);
  __builtin_amdgcn_sched_barrier(0);
  // ---- L3 s0 + T2 s1 (5 outputs padded to one 16-wide tile)
  zX = *reinterpret_cast<const f32x4*>(bias + 2 * kH + 4 * gq);
  zY = zX;
  zX = layer3(w3.s[0], cx0, zX);
  zY = layer3(w3.s[0], cy0, zY);
  cx1 = tanh_split(accX[2], accX[3]);
  cy1 = tanh_split(accY[2], accY[3]);
  __builtin_amdgcn_sched_barrier(0);
  // ---- L3 s1
  zX = layer3(w3.s[1], cx1, zX);
  zY = layer3(w3.s[1], cy1, zY);
  __builtin_amdgcn_s_setprio(0);
}

// This lane's 8 layer-1 inputs of row j for one K slice (see policy_core): columns 8 (gq & 1) .. + 7, or, with
// 17..64 inputs, columns 32 slice + 8 gq .. + 7 with zeros beyond the row's D columns (what lies there is the
// next row).
template <typename S>
__device__ __forceinline__ void load_row_inputs(const float* __restrict__ rows, int j, int gq, int slice, float (&v)[8]) {
  constexpr int D = S::D;
  const int c0 = 32 * slice + (S::kWideIn ? 8 * gq : 8 * (gq & 1));
  // rows are D*4 bytes apart (a multiple of 8, not of 16): read as float2
  const float2* src = reinterpret_cast<const float2*>(rows + j * D + c0);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float2 x = src[q];
    if constexpr (S::kWideIn) {
      if (c0 + 2 * q >= D) x = make_float2(0.0f, 0.0f);
    }
    v[2 * q] = x.x;
    v[2 * q + 1] = x.y;
  }
}

template <typename S, bool VALUE = false>
__device__ __forceinline__ void policy_pair(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                            const W3Terms& w3, float* __restrict__ rowsX,
                                            float* __restrict__ rowsY, int lane,
                                            float* __restrict__ valX = nullptr, float* __restrict__ valY = nullptr) {
  constexpr int D = S::D;
  const int j = lane & 15, gq = lane >> 4;
  float vx[S::kSlices1][8], vy[S::kSlices1][8];
#pragma unroll
  for (int s = 0; s < S::kSlices1; ++s) {
    load_row_inputs<S>(rowsX, j, gq, s, vx[s]);
    load_row_inputs<S>(rowsY, j, gq, s, vy[s]);
  }
  f32x4 zX, zY;
  policy_core<S>(wsm, bias, w3, vx, vy, zX, zY, lane);
  if constexpr (VALUE) {
    // output 0: lane group 0; row-term layout: its three term rows, otherwise register 0
    if (gq == 0) {
      valX[j] = S::kRowTerms ? (zX[0] + zX[1]) + zX[2] : zX[0];
      valY[j] = S::kRowTerms ? (zY[0] + zY[1]) + zY[2] : zY[0];
    }
  } else if constexpr (S::kRowTerms) {
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
template <typename S>
__global__ void pack_bf16_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                 const float* __restrict__ b1, const float* __restrict__ W2,
                                 const float* __restrict__ b2, const float* __restrict__ W3,
                                 const float* __restrict__ b3, int nout) {
  using PkB = PkT<true, S::kWideIn, S::kSlices1>;
  constexpr int D = S::D, KIN = S::KIN, KS1 = S::kSlices1;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * PkB::RUN_BYTES;
  W1 += size_t(run) * D * kH;
  b1 += size_t(run) * kH;
  W2 += size_t(run) * kH * kH;
  b2 += size_t(run) * kH;
  W3 += size_t(run) * kH * nout;
  b3 += size_t(run) * nout;
  constexpr int n1 = 4 * KS1 * 64 * 8, n2 = 4 * 2 * 64 * 8, n3 = 2 * 64 * 8, nb = 2 * kH + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n1) {   // [m][s][lane][e]; k = 8 gq + e for gq < 2, zero above (all four lane groups when kWideIn)
    const int e = idx % 8, lane = (idx / 8) % 64, sl = (idx / 512) % KS1, m = idx / (512 * KS1);
    const int gq = lane / 16, k = 32 * sl + 8 * gq + e, o = 16 * m + lane % 16;
    reinterpret_cast<uint16_t*>(out + PkB::OFF_W1A)[idx] = f32_to_bf16_rne(((gq < 2 || S::kWideIn) && k < KIN) ? W1[size_t(k) * kH + o] : 0.0f);
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
template <typename S, bool VALUE = false>
__device__ __forceinline__ void policy_pair_bf(const uint8_t* __restrict__ wsm, const float* __restrict__ bias,
                                               const W3Terms& w3, float* __restrict__ rowsX,
                                               float* __restrict__ rowsY, int lane,
                                               float* __restrict__ valX = nullptr, float* __restrict__ valY = nullptr) {
  constexpr int D = S::D;
  const int j = lane & 15, gq = lane >> 4;
  __builtin_amdgcn_s_setprio(2);   // see policy_core
  {
    uint32_t zero = 0;   // see policy_pair: keeps the LDS weight reads inside the step loop
    asm volatile("" : "+v"(zero));
    wsm += zero;
    bias += zero;
  }
  using PkB = PkT<true, S::kWideIn, S::kSlices1>;
  constexpr int KS1 = S::kSlices1;
  const bf16x8* w1 = reinterpret_cast<const bf16x8*>(wsm + PkB::OFF_W1A);  // [m][slice][lane]
  const bf16x8* w2 = reinterpret_cast<const bf16x8*>(wsm + PkB::OFF_W2A);  // [m][s][lane]
  // layer-1 B operands: inputs 8 (gq & 1) .. + 7 of the row, lane groups 2, 3 meet zero weights; with
  // 17..32 inputs, inputs 8 gq .. + 7
  bf16x8 bx[KS1], by[KS1];
#pragma unroll
  for (int s = 0; s < KS1; ++s) {
    float vx[8], vy[8];
    load_row_inputs<S>(rowsX, j, gq, s, vx);
    load_row_inputs<S>(rowsY, j, gq, s, vy);
    u32x4 px, py;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      px[q] = pack_bf16_rne(vx[2 * q], vx[2 * q + 1]);
      py[q] = pack_bf16_rne(vy[2 * q], vy[2 * q + 1]);
    }
    bx[s] = __builtin_bit_cast(bf16x8, px);
    by[s] = __builtin_bit_cast(bf16x8, py);
  }
  f32x4 accX[4], accY[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    accX[m] = *reinterpret_cast<const f32x4*>(bias + 16 * m + 4 * gq);
    accY[m] = accX[m];
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
#pragma unroll
    for (int s = 0; s < KS1; ++s) {
      const bf16x8 a = w1[(m * KS1 + s) * 64 + lane];
      accX[m] = MPE_MFMA_BF(a, bx[s], accX[m]);
      accY[m] = MPE_MFMA_BF(a, by[s], accY[m]);
    }
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
  __builtin_amdgcn_s_setprio(0);
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

}  // namespace

}  // namespace mpe
