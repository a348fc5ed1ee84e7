"""libjigsaw_decode: MI355X-native paged decode attention for ragged, long-tailed rollout batches.

`binding` wraps the C ABI (include/jigsaw_decode.h); `workloads` generates the seeded synthetic
decode steps used by the tests and the benchmark; `build` compiles the HIP library in-tree.
"""
