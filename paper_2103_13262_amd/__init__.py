"""MI355X-native single-GPU Mixture-of-Experts layer (forward + backward).

`paper_2103_13262_amd.binding` is the thin ctypes layer over libmoe355.so (the
C ABI declared in include/moe355.h); `paper_2103_13262_amd.synth` makes the
seeded synthetic workloads.  Nothing is imported eagerly so that the input
generator can be used without the HIP library.
"""
__all__ = ["binding", "synth", "build"]
