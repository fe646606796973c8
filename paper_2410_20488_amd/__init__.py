"""MI355X-native FIRP decoding step: HIP kernels behind a C-ABI library, plus a thin binding."""
