"""MI355X-native Elman RNN language-model training step (hand-written HIP behind a C ABI)."""
