"""k-means-quantised GEMV / small-batch GEMM for AMD MI355X (gfx950).

``paper_2602_15563_amd.kmq`` is the thin binding over the C-ABI library
(include/kmq.h); ``paper_2602_15563_amd.synth`` generates seeded synthetic
inputs.  Nothing is imported eagerly so that the input generator can be used
on a machine without the built library.
"""
__all__ = ["kmq", "synth"]
