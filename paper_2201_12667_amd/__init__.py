"""MI355X-native SLIDE training step: HIP kernels behind a C ABI, plus a thin binding."""
