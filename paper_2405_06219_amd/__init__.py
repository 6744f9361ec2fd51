"""MI355X-native SKVQ hot path (arXiv 2405.06219): quantize-on-evict and decode attention
over a 2-bit / 1.5-bit KV cache with an fp16 sliding window, as hand-written HIP kernels
behind a C ABI (include/skvq.h).  `binding` is the thin ctypes layer; `synth` draws the
seeded synthetic workloads."""
