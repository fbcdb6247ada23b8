"""MI355X-native HyLRA decode-attention hot path (hand-written HIP behind a C ABI)."""
