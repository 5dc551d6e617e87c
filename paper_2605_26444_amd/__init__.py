"""MI355X-native NanoSpec draft-step hot path: thin Python binding over libnanospec.so.

`paper_2605_26444_amd.binding` mirrors the C ABI of include/nanospec.h; `synth` makes the seeded
synthetic inputs; `build` compiles the HIP library in-tree.  Nothing here computes on the CPU.
"""
