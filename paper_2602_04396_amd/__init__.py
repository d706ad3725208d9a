"""MI355X-native LoRDO optimizer hot path (HIP kernels behind a C ABI)."""
