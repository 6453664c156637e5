"""MI355X-native batched MPE simple-spread rollout (HIP kernels behind a C ABI)."""
