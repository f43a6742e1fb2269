"""MI355X-native VScan token reduction: HIP kernels behind a C ABI plus a thin binding."""
