"""MI355X-native hot path of the PaFu-KV chunk step (score, select, compact, attention).

The compute lives in libpafu.so (hand-written HIP for gfx950 behind a C ABI, see
include/pafu.h); `binding` marshals torch tensors into it and `workloads` draws the
seeded synthetic inputs.  Nothing here computes on the CPU.
"""
