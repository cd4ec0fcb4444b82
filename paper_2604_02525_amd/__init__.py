"""MI355X-native AdaHOP per-GEMM hot path: HIP kernels behind a C ABI plus a thin ctypes binding."""
