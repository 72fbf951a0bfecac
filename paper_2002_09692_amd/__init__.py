"""MI355X-native kernels for one SAPS-PSGD round (sparsified peer exchange fused with the local step).

`paper_2002_09692_amd.binding` wraps the C ABI of include/saps.h (needs the built libsaps.so and a GPU);
`paper_2002_09692_amd.synth` generates the seeded synthetic workloads; `paper_2002_09692_amd.build`
compiles the library.  Nothing is imported eagerly so that the generators work without a GPU.
"""
__all__ = ["binding", "build", "synth"]
