"""MI355X-native MoE-layer forward of Pipeline MoE (one device's share): HIP kernels behind a C ABI."""
