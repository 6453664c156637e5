// Stand-alone probe: which store patterns reach which HBM write rate on one MI355X.
//
// The env-only rollout is bound by trajectory stores whose addresses are fixed by the trajectory
// layout [T][E][N][D]: a group of 64 envs owns one contiguous 13,824-byte piece of every time slice.
// This probe writes a buffer of the rollout's size with plain 16-byte stores in several patterns and
// times each with HIP events, to separate what the memory system allows for THAT address pattern from
// what it allows for a free choice of addresses:
//   sweep   - grid-stride: at every instant all wavefronts together cover one contiguous window
//   short   - many short-lived 256-thread blocks, 16 bytes per thread (what library fills do)
//   blocked - like sweep, but each wavefront owns R consecutive KiB of the window per iteration
//   rollout - persistent groups, one contiguous chunk per group and time slice (the rollout's pattern),
//             with the real 54-float rows (obs only) and with rows padded to 64 floats, plain and
//             nontemporal stores
//   small   - the rollout's pattern with 64-byte rows plus the small outputs of every step (4-byte reward
//             and 1-byte action per row, 1-byte done flag per 4 rows) written per lane: what the small
//             partial-line outputs cost, and what nontemporal row stores change about it
// Build: python -m paper_2311_10090_amd.build --probe ; run: paper_2311_10090_amd/store_pattern_probe
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ void sweep_kernel(v4f* out, size_t n16) {
  v4f v = {1.f, 2.f, 3.f, (float)threadIdx.x};
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) out[i] = v;
}

__global__ void short_kernel(v4f* out, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) out[i] = v4f{1.f, 2.f, 3.f, (float)blockIdx.x};
}

// per iteration the grid covers one contiguous window; wavefront s of block b writes its own R KiB of it
__global__ void blocked_kernel(v4f* out, size_t n16, int R) {
  const int lane = threadIdx.x & 63, s = threadIdx.x >> 6, wpb = blockDim.x >> 6;
  const size_t piece16 = (size_t)wpb * R * 64, window16 = piece16 * gridDim.x;
  v4f v = {1.f, 2.f, 3.f, (float)blockIdx.x};
  for (size_t base = (size_t)blockIdx.x * piece16; base + piece16 <= n16; base += window16)
    for (int r = 0; r < R; ++r) out[base + ((size_t)s * R + r) * 64 + lane] = v;
}

// block g owns [g*chunk16, (g+1)*chunk16) of each of T slices
template <bool NT>
__global__ void rollout_kernel(v4f* out, int chunk16, size_t slice16, int T) {
  v4f v = {1.f, 2.f, 3.f, (float)blockIdx.x};
  v4f* p = out + (size_t)blockIdx.x * chunk16;
  for (int t = 0; t < T; ++t) {
    for (int j = threadIdx.x; j < chunk16; j += blockDim.x) {
      if (NT) __builtin_nontemporal_store(v, &p[j]); else p[j] = v;
    }
    p += slice16;
  }
}

// 256-thread blocks; wavefront w of block b owns rows [(4b + w) * 64, +64) of each slice: 64 bytes of
// observation per row, and with SMALL a 4-byte reward and a 1-byte action per row and a 1-byte done flag
// per 4 rows, each in an array of its own.  `rows` must be gridDim.x * 256.
template <bool SMALL, bool NT>
__global__ __launch_bounds__(256) void small_outputs_kernel(v4f* obs, float* rew, uint8_t* act, uint8_t* done,
                                                             size_t rows, int T) {
  const int lane = threadIdx.x & 63;
  const size_t row0 = ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 64;
  v4f v = {1.f, 2.f, 3.f, (float)blockIdx.x};
  for (int t = 0; t < T; ++t) {
    v4f* o = obs + ((size_t)t * rows + row0) * 4;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (NT) __builtin_nontemporal_store(v, &o[k * 64 + lane]); else o[k * 64 + lane] = v;
    }
    if (SMALL) {
      rew[(size_t)t * rows + row0 + lane] = v.x;
      act[(size_t)t * rows + row0 + lane] = (uint8_t)lane;
      if ((lane & 3) == 0) done[(size_t)t * (rows / 4) + row0 / 4 + lane / 4] = 0;
    }
  }
}

int main() {
  const int E = 65536, T = 128;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { printf("no device\n"); return 1; }
  const size_t cap16 = (size_t)E * 64 / 4 * T;   // 2 GiB: the padded-row case
  v4f* buf;
  if (hipMalloc(&buf, cap16 * 16) != hipSuccess) { printf("allocation failed\n"); return 1; }
  bool ok = true;
  auto run = [&](const char* name, size_t n16, auto launch) {
    if (!ok) return;
    for (int i = 0; i < 3; i++) launch();
    if (hipDeviceSynchronize() != hipSuccess) { printf("%s: launch failed\n", name); ok = false; return; }
    float sum = 0, best = 1e9f;
    for (int i = 0; i < 10; i++) {
      (void)hipEventRecord(a); launch(); (void)hipEventRecord(b); (void)hipEventSynchronize(b);
      float ms = 0; (void)hipEventElapsedTime(&ms, a, b); sum += ms; best = ms < best ? ms : best;
    }
    printf("%-50s avg %.4f ms  min %.4f ms  %5.0f GB/s\n", name, sum / 10, best, n16 * 16 / (sum / 10 * 1e-3) / 1e9);
    fflush(stdout);
  };
  char nm[96];
  const size_t slice54 = (size_t)E * 54 / 4, n54 = slice54 * T;   // the rollout's observation bytes
  const size_t slice64 = (size_t)E * 64 / 4, n64 = slice64 * T;
  for (int blocks : {256, 1024, 2048}) {
    snprintf(nm, sizeof nm, "sweep, %d blocks x 256 threads", blocks);
    run(nm, n54, [&] { hipLaunchKernelGGL(sweep_kernel, dim3(blocks), dim3(256), 0, 0, buf, n54); });
  }
  run("short blocks, 256 threads x 16 B", n54, [&] { hipLaunchKernelGGL(short_kernel, dim3((unsigned)((n54 + 255) / 256)), dim3(256), 0, 0, buf, n54); });
  run("hipMemsetAsync", n54, [&] { (void)hipMemsetAsync(buf, 1, n54 * 16, 0); });
  for (int R : {1, 2, 4, 8, 16}) {
    snprintf(nm, sizeof nm, "blocked, 256 blocks x 256 threads, R = %d KiB", R);
    run(nm, n64, [&] { hipLaunchKernelGGL(blocked_kernel, dim3(256), dim3(256), 0, 0, buf, n64, R); });
  }
  for (int thr : {64, 128}) {
    snprintf(nm, sizeof nm, "rollout, 1024 groups x %d threads, 54-float rows", thr);
    run(nm, n54, [&] { hipLaunchKernelGGL(rollout_kernel<false>, dim3(1024), dim3(thr), 0, 0, buf, (int)(slice54 / 1024), slice54, T); });
  }
  run("rollout, 256 groups x 256 threads, 54-float rows", n54, [&] { hipLaunchKernelGGL(rollout_kernel<false>, dim3(256), dim3(256), 0, 0, buf, (int)(slice54 / 256), slice54, T); });
  run("rollout, 1024 groups x 64 threads, 64-float rows", n64, [&] { hipLaunchKernelGGL(rollout_kernel<false>, dim3(1024), dim3(64), 0, 0, buf, (int)(slice64 / 1024), slice64, T); });
  run("rollout, 1024 x 64, 54-float rows, nontemporal", n54, [&] { hipLaunchKernelGGL(rollout_kernel<true>, dim3(1024), dim3(64), 0, 0, buf, (int)(slice54 / 1024), slice54, T); });
  run("rollout, 1024 x 64, 64-float rows, nontemporal", n64, [&] { hipLaunchKernelGGL(rollout_kernel<true>, dim3(1024), dim3(64), 0, 0, buf, (int)(slice64 / 1024), slice64, T); });
  // small outputs: 262,144 rows x 128 slices; the GB/s column counts the 64-byte rows only
  const size_t rows = (size_t)1024 * 256, nrow16 = rows * 4 * T;
  float* rew = nullptr; uint8_t *act = nullptr, *done = nullptr;
  if (hipMalloc(&rew, rows * 4 * T) != hipSuccess || hipMalloc(&act, rows * T) != hipSuccess ||
      hipMalloc(&done, rows / 4 * T) != hipSuccess) { printf("allocation failed\n"); return 1; }
  run("small: rows only", nrow16, [&] { hipLaunchKernelGGL((small_outputs_kernel<false, false>), dim3(1024), dim3(256), 0, 0, buf, rew, act, done, rows, T); });
  run("small: rows + small outputs", nrow16, [&] { hipLaunchKernelGGL((small_outputs_kernel<true, false>), dim3(1024), dim3(256), 0, 0, buf, rew, act, done, rows, T); });
  run("small: nontemporal rows only", nrow16, [&] { hipLaunchKernelGGL((small_outputs_kernel<false, true>), dim3(1024), dim3(256), 0, 0, buf, rew, act, done, rows, T); });
  run("small: nontemporal rows + small outputs", nrow16, [&] { hipLaunchKernelGGL((small_outputs_kernel<true, true>), dim3(1024), dim3(256), 0, 0, buf, rew, act, done, rows, T); });
  (void)hipFree(buf); (void)hipFree(rew); (void)hipFree(act); (void)hipFree(done);
  return ok ? 0 : 1;
}
