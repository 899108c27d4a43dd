"""MI355X-native GraphKV eviction pass: HIP kernels behind a C ABI (include/graphkv.h)
and a thin Python binding.  `synth` holds the seeded input generators."""
