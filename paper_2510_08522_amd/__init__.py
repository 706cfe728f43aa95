"""MI355X-native gradient aggregate + statistics hot path (HIP kernels behind a C ABI)."""
