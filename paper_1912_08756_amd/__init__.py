"""MI355X-native query-time path of Interleaved Composite Quantization.

`binding` wraps the C-ABI library built from `csrc/` (names follow
include/icq.h); `synth` draws seeded synthetic workloads.  Nothing here falls
back to a CPU implementation: calling a binding without the built HIP library
raises.
"""
