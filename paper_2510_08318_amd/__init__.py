"""MI355X-native non-causal linear attention (Hedgehog feature map) -- HIP kernels behind a C ABI."""
