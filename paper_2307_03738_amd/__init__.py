"""MI355X-native group-quantized GEMV / small-M GEMM (2/3/4-bit codes, per-group scale and
zero-point).  `binding` wraps the C-ABI library built from csrc/; `synth` draws the seeded
benchmark inputs.  Nothing is loaded at import time."""
