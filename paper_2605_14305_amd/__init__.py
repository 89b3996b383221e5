"""MI355X-native FeF-DLLM speculative verify step: thin Python binding over the C-ABI
library built from ``csrc/`` (hand-written HIP kernels for gfx950)."""
