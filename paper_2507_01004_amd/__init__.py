"""MI355X-native ZeCO hot path: chunkwise GLA segment forward, segment-state scan and
initial-state correction as hand-written HIP kernels behind a C ABI (see include/zeco.h).

`paper_2507_01004_amd.zeco`  - the binding (loads csrc/libzeco.so; fails loudly if it is missing)
`paper_2507_01004_amd.synth` - seeded synthetic workloads
"""
