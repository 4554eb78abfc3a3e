"""MI355X-native PBS-Attn prefill path (hand-written HIP kernels behind a C-ABI library)."""
