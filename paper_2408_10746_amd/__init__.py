"""MI355X-native cached Parallel-Adapter training step (HIP kernels behind a C ABI)."""
