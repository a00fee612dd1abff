"""MI355X-native Persistent Block-Sparse Attention (PBSA) decode path: HIP kernels behind a C ABI."""
