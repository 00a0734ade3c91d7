"""MI355X-native CQIL group forward: HIP kernels behind a C-ABI library plus a thin binding."""
