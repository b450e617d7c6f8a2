"""MI355X-native BitLinear W1.58A8 (BitNet b1.58, arXiv 2402.17764, Section 2).

The product lives in a C-ABI shared library of hand-written HIP kernels for gfx950
(csrc/, declared in include/bitnet.h).  `paper_2402_17764_amd.binding` is a thin ctypes layer
with the same names; it loads the library lazily and raises if it is missing.  `synth` holds
the seeded input generators and no arithmetic of the method.
"""
__all__ = ["binding", "synth", "build"]
