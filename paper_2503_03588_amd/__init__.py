"""MI355X-native PowerAttention hot path: a C-ABI library of HIP kernels plus a thin binding."""
