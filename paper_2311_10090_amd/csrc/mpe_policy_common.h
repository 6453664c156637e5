// Shared pieces of the fused-rollout kernels: packed weight layouts, the pack kernel, tanh,
// wavefront-level LDS fence, Gumbel-max sampling.
#pragma once

#include "mpe_launch.h"

namespace mpe {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__host__ __device__ constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }

template <int N, int H, bool BF16>
struct Shape {
  static_assert(BF16 || 4 * N + 2 <= 16, "fp32 layout: layer 1 reads 16 inputs per row");
  static constexpr int D = 6 * N;
  static constexpr int KIN = 4 * N + 2;           // non-zero leading entries of an observation
  static constexpr int KS = BF16 ? 32 : 4;        // K extent of one MFMA
  static constexpr int MT = H / 16;               // 16-wide tiles of hidden units
  static constexpr int S1 = BF16 ? cdiv(KIN, KS) : 4;  // K slices of layer 1 (fp32: always 16 inputs, zero padded)
  static constexpr int S2 = H / KS;               // K slices of layers 2 and 3
  static constexpr int ELT = BF16 ? 2 : 4;        // bytes per weight
  static constexpr int LANE_ELTS = BF16 ? 8 : 1;  // A-operand elements one lane holds per MFMA
  // packed buffer sections (bytes), all multiples of 16
  static constexpr size_t W1A_BYTES = size_t(MT) * S1 * 64 * LANE_ELTS * ELT;
  static constexpr size_t W2A_BYTES = size_t(MT) * S2 * 64 * LANE_ELTS * ELT;
  static constexpr size_t W3A_BYTES = size_t(S2) * 64 * LANE_ELTS * ELT;
  static constexpr size_t BIAS_BYTES = size_t(2 * H + 16) * 4;
  static constexpr size_t OFF_W1A = 0;
  static constexpr size_t OFF_W2A = OFF_W1A + W1A_BYTES;
  static constexpr size_t OFF_W3A = OFF_W2A + W2A_BYTES;
  static constexpr size_t OFF_BIAS = OFF_W3A + W3A_BYTES;
  static constexpr size_t RUN_BYTES = OFF_BIAS + BIAS_BYTES;
};

// Hidden unit that K position (slice s, lane group gq, element e) of layers 2/3 refers to:
// the accumulator register (tile m, r) of lane group gq holds unit 16m + 4gq + r.
template <bool BF16>
__host__ __device__ constexpr int hidden_of(int s, int gq, int e) {
  return BF16 ? (32 * s + 16 * (e / 4) + 4 * gq + (e % 4)) : (16 * (s / 4) + 4 * gq + (s % 4));
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// One thread per packed element of one run.
template <int N, int H, bool BF16>
__global__ void pack_policy_kernel(uint8_t* __restrict__ packed, const float* __restrict__ W1,
                                   const float* __restrict__ b1, const float* __restrict__ W2,
                                   const float* __restrict__ b2, const float* __restrict__ W3,
                                   const float* __restrict__ b3) {
  using S = Shape<N, H, BF16>;
  const int run = blockIdx.y;
  uint8_t* out = packed + size_t(run) * S::RUN_BYTES;
  W1 += size_t(run) * S::D * H;
  b1 += size_t(run) * H;
  W2 += size_t(run) * H * H;
  b2 += size_t(run) * H;
  W3 += size_t(run) * H * kNumActions;
  b3 += size_t(run) * kNumActions;
  const int n1 = S::MT * S::S1 * 64 * S::LANE_ELTS;
  const int n2 = S::MT * S::S2 * 64 * S::LANE_ELTS;
  const int n3 = S::S2 * 64 * S::LANE_ELTS;
  const int nb = 2 * H + 16;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  auto put = [&](size_t off, int i, float v) {
    if (BF16) reinterpret_cast<uint16_t*>(out + off)[i] = f32_to_bf16_rne(v);
    else reinterpret_cast<float*>(out + off)[i] = v;
  };
  // fp32: the pre-activations of both tanh layers are produced already multiplied by
  // 2*log2(e), so tanh(x) = 1 - 2 / (2^y + 1) needs no multiply in the kernel.
  const float pre = BF16 ? 1.0f : 2.0f * kLog2e;
  if (idx < n1) {
    int m, s, lane, e;
    if (BF16) {  // [m][s][lane][e]
      e = idx % 8; lane = (idx / 8) % 64; s = (idx / 512) % S::S1; m = idx / (512 * S::S1);
    } else {     // [m][lane][s]: one 16-byte read gives a lane its S1 = 4 slices
      s = idx % S::S1; lane = (idx / S::S1) % 64; m = idx / (S::S1 * 64); e = 0;
    }
    // lane (i = lane%16, gq = lane/16) ; k = KS*s + LANE_ELTS*gq + e (natural order)
    const int k = S::KS * s + S::LANE_ELTS * (lane / 16) + e;
    const int o = 16 * m + lane % 16;
    put(S::OFF_W1A, idx, k < S::KIN ? pre * W1[size_t(k) * H + o] : 0.0f);
    return;
  }
  idx -= n1;
  if (idx < n2) {
    int m, s, lane, e;
    if (BF16) {  // [m][s][lane][8]
      e = idx % 8; lane = (idx / 8) % 64; s = (idx / 512) % S::S2; m = idx / (512 * S::S2);
    } else {     // [m][s/4][lane][s%4]
      const int s_lo = idx % 4; lane = (idx / 4) % 64; const int s_hi = (idx / 256) % (S::S2 / 4);
      m = idx / (256 * (S::S2 / 4)); s = 4 * s_hi + s_lo; e = 0;
    }
    const int k = hidden_of<BF16>(s, lane / 16, e);
    put(S::OFF_W2A, idx, pre * W2[size_t(k) * H + 16 * m + lane % 16]);
    return;
  }
  idx -= n2;
  if (idx < n3) {
    int s, lane, e;
    if (BF16) { e = idx % 8; lane = (idx / 8) % 64; s = idx / 512; }
    else { const int s_lo = idx % 4; lane = (idx / 4) % 64; s = 4 * (idx / 256) + s_lo; e = 0; }
    const int k = hidden_of<BF16>(s, lane / 16, e);
    const int o = lane % 16;
    put(S::OFF_W3A, idx, o < kNumActions ? W3[size_t(k) * kNumActions + o] : 0.0f);
    return;
  }
  idx -= n3;
  if (idx < nb) {
    float v;
    if (idx < H) v = pre * b1[idx];
    else if (idx < 2 * H) v = pre * b2[idx - H];
    else v = (idx - 2 * H) < kNumActions ? b3[idx - 2 * H] : 0.0f;
    reinterpret_cast<float*>(out + S::OFF_BIAS)[idx] = v;
  }
}

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
