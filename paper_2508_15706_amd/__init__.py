"""MI355X-native SparseLoCo compress + aggregate path (HIP kernels behind a C ABI)."""
