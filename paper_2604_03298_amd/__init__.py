"""MI355X-native ENEC lossless bf16 weight codec (hand-written HIP behind a C ABI)."""
