"""FP4 (E2M1) quantized linear layer, forward and backward, for MI355X (gfx950).

The compute lives in hand-written HIP kernels behind a C ABI (include/fp4_linear.h);
`paper_2501_17116_amd.binding` marshals torch device tensors into those calls.
Importing this package does not load the native library; the first call does, and it
raises if the library has not been built.
"""
__all__ = ["binding", "synth"]
