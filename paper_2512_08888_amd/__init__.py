"""MI355X-native multi-orientation (rotation-invariant) convolution.

The product is the C-ABI library built from csrc/ (HIP, gfx950) and declared in
include/rotconv.h; `binding` is the thin ctypes layer over it and `synth` the
seeded input generators.  Nothing is imported eagerly so that `synth` can be
used on machines without the HIP runtime.
"""
__all__ = ["binding", "synth"]
