// Stand-alone probe (not part of libmpe): how far do matrix (MFMA) and vector instructions of the
// fused kernels' instruction mix overlap on this chip?  One block per CU; per iteration a wavefront
// runs 24 independent v_mfma_f32_16x16x32_bf16 and/or 16 tanh evaluations (mul, exp2, add, rcp, fma),
// (a) as two bursts, (b) finely interleaved (one matrix instruction, then ~3 vector instructions),
// with one or two wavefronts per SIMD; also the vector work split into its full-rate and its
// transcendental part.  Prints cycles per iteration assuming 2.4 GHz (only the ratios matter).
// Build and run:  python -m paper_2311_10090_amd.build --probe && paper_2311_10090_amd/coexec_probe
#include <hip/hip_runtime.h>
#include <cstdio>
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0)
__device__ __forceinline__ float act(float x) {   // mul, exp2, add, rcp, fma
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(x * 2.885f) + 1.0f), 1.0f);
}
__device__ __forceinline__ float act_simple(float x) {   // five full-rate instructions
  x = fmaf(x, 0.999f, 0.001f); x = fmaf(x, 0.998f, 0.002f); x = fmaf(x, 0.997f, 0.003f); x = fmaf(x, 0.996f, 0.004f);
  return fmaf(x, 0.995f, 0.005f);
}
__device__ __forceinline__ float act_trans(float x) {    // two transcendental instructions
  return __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(x));
}
template <int MODE>
__global__ __launch_bounds__(512) void k(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(0.01f * (lane + e)); b[e] = (__bf16)(0.02f * (lane - e)); }
  f32x4 acc[6];
  for (int i = 0; i < 6; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = 0.001f * (lane + i);
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0 || MODE == 2) {       // burst of 24 matrix instructions
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 6; ++i) acc[i] = MFMA(a, b, acc[i]);
    }
    if (MODE == 2) __builtin_amdgcn_sched_barrier(0);
    if (MODE == 1 || MODE == 2) {       // burst of 16 activations = 80 vector instructions (32 transcendental)
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = act(v[i]);
    }
    if (MODE == 2) __builtin_amdgcn_sched_barrier(0);
    if (MODE == 4 || MODE == 6) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 6; ++i) acc[i] = MFMA(a, b, acc[i]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE == 4 || MODE == 5) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = act_simple(v[i]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE == 6 || MODE == 7) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = act_trans(v[i]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE == 3) {                    // fine interleave: 1 matrix instruction, then 2/3 of an activation
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 6; ++i) {
          acc[i] = MFMA(a, b, acc[i]);
          __builtin_amdgcn_sched_barrier(0);
          const int q = (r * 6 + i) * 2 / 3;            // 24 slots -> 16 activations
          if ((r * 6 + i) * 2 % 3 != 2 && q < 16) v[q] = act(v[q]);
          __builtin_amdgcn_sched_barrier(0);
        }
    }
  }
  float s = 0;
  for (int i = 0; i < 6; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  for (int i = 0; i < 16; ++i) s += v[i];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}
template <int MODE>
float run(float* d, int threads, int iters) {
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipLaunchKernelGGL(k<MODE>, dim3(256), dim3(threads), 0, 0, d, 10);
  hipEventRecord(e0);
  hipLaunchKernelGGL(k<MODE>, dim3(256), dim3(threads), 0, 0, d, iters);
  hipEventRecord(e1); hipEventSynchronize(e1);
  float ms; hipEventElapsedTime(&ms, e0, e1); return ms;
}
int main() {
  float* d; hipMalloc(&d, 256 * 512 * 4);
  const int iters = 20000;
  for (int threads : {256, 512}) {
    float m0 = run<0>(d, threads, iters), m1 = run<1>(d, threads, iters), m2 = run<2>(d, threads, iters), m3 = run<3>(d, threads, iters);
    const double cyc = 2.4e6 / iters;   // cycles per iteration per ms
    printf("waves/SIMD %d: matrix only %.0f cyc/iter, vector only %.0f, bursts %.0f, fine interleave %.0f\n",
           threads / 256, m0 * cyc, m1 * cyc, m2 * cyc, m3 * cyc);
    float m4 = run<4>(d, threads, iters), m5 = run<5>(d, threads, iters), m6 = run<6>(d, threads, iters), m7 = run<7>(d, threads, iters);
    printf("   simple only (80 fma) %.0f, matrix + simple %.0f; transcendental only (32) %.0f, matrix + transcendental %.0f\n",
           m5 * cyc, m4 * cyc, m7 * cyc, m6 * cyc);
  }
  return 0;
}
