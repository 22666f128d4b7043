"""MI355X (gfx950) implementation of the quantized linear-layer hot path of SNIP
(arXiv 2602.01410): block-scaled FP8/FP4 quantization, the three GEMMs of a linear layer on
scaled MFMA, and the quantization-error statistics pass.

``snip`` is the ctypes binding of the C-ABI library (``include/snip.h``); ``workloads``
holds the seeded synthetic inputs.  Importing the package does not load the HIP library;
the first call into ``snip`` does, and raises if it has not been built.
"""
__all__ = ["workloads", "snip"]
