"""MI355X-native AT-GRPO policy-loss hot path (HIP kernels behind a C ABI)."""
