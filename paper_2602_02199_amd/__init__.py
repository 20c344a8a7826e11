"""MI355X-native LASER-KV block-wise prefill KV selection (HIP kernels behind a C-ABI)."""
