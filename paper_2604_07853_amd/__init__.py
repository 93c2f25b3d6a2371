"""MI355X-native hot path of QaRL: low-bit quantized MoE expert GEMM, weight quantizer,
top-k router and per-token log-prob comparison, as hand-written HIP behind a C ABI."""
