"""MI355X-native kernels for the computation GuidedQuant adds to layer-wise PTQ:
averaged squared output gradients, grouped Fisher Gram blocks and the layer
objective.  The compute lives in libgq.so (HIP, gfx950); this package only
binds its C ABI."""

__all__ = ["binding", "workloads", "build"]
