"""MI355X-native DyMoE mixed-precision MoE layer (hand-written HIP behind a C ABI).

`paper_2603_19172_amd.binding` loads the compiled library and exposes its entry
points; `paper_2603_19172_amd.synth` draws the seeded synthetic workloads.
Importing the package itself loads nothing.
"""
__all__ = ["binding", "synth"]
