"""MI355X-native KNN-SSD self-speculative decoding hot path (HIP kernels behind a C ABI)."""
