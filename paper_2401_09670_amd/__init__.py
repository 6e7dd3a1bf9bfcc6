"""MI355X-native prefill / KV-migrate / decode hot path (HIP kernels behind a C ABI)."""
