"""MI355X-native Cerberus verify step: HIP kernels behind a C ABI, plus a thin binding."""
