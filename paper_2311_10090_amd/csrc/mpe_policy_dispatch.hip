// Routing of mpe_set_policy / mpe_rollout to the kernel family that is built for the shape.
#include "mpe_launch.h"

namespace mpe {

hipError_t ensure_policy_bytes(PolicyBuffers& pb, size_t bytes) {
  if (pb.bytes >= bytes) return hipSuccess;
  if (pb.borrowed) return hipErrorOutOfMemory;   // the caller sized it with packed_policy_bytes
  if (pb.packed) {
    hipError_t e = hipFree(pb.packed);
    if (e != hipSuccess) return e;
    pb.packed = nullptr;
    pb.bytes = 0;
  }
  hipError_t e = hipMalloc(&pb.packed, bytes);
  if (e != hipSuccess) return e;
  pb.bytes = bytes;
  return hipSuccess;
}

void free_policy(PolicyBuffers& pb) {
  if (pb.packed && !pb.borrowed) (void)hipFree(pb.packed);
  pb.packed = nullptr;
  pb.bytes = 0;
}

static const char* kUnsupported =
    "unsupported policy shape: need (num_agents, hidden, dtype) in {(1..3, 64, fp32 or bf16), (4..10, 64, fp32), "
    "(4..10, 64 | 128, bf16)}";

size_t packed_policy_bytes(int N, int H, int R, int weight_dtype) {
  if (weight_dtype == 1 && wide_supported(N, H)) return size_t(R) * packed_run_bytes_wide(N, H);
  if (f32_supported(N, H, weight_dtype == 1)) return size_t(R) * packed_run_bytes_f32(N, weight_dtype == 1);
  return 0;
}

hipError_t pack_policy(PolicyBuffers& pb, int N, int H, int R, int weight_dtype, const float* W1,
                       const float* b1, const float* W2, const float* b2, const float* W3,
                       const float* b3, hipStream_t s, const char** why) {
  if (weight_dtype == 1 && wide_supported(N, H)) return pack_policy_wide(pb, N, H, R, W1, b1, W2, b2, W3, b3, 5, s);
  if (f32_supported(N, H, weight_dtype == 1)) return pack_policy_f32(pb, N, R, W1, b1, W2, b2, W3, b3, 5, weight_dtype == 1, s);
  *why = kUnsupported;
  return hipSuccess;
}

hipError_t launch_rollout_policy(int N, int H, int weight_dtype, const RolloutArgs& A,
                                 const PolicyBuffers& pb, hipStream_t s, const char** why) {
  if (weight_dtype == 1 && wide_supported(N, H)) return launch_rollout_policy_wide(N, H, A, pb, s, why);
  if (f32_supported(N, H, weight_dtype == 1)) return launch_rollout_policy_f32(N, weight_dtype == 1, A, pb, s, why);
  *why = kUnsupported;
  return hipSuccess;
}

}  // namespace mpe
