"""MI355X-native hot path of one mixed-precision training step (arXiv 1710.03740).

The work is done by hand-written HIP kernels behind a C ABI (include/mpt.h,
built into libmpt.so); `paper_1710_03740_amd.binding` marshals arguments to it.
There is no CPU fallback: using the binding without the built library raises.
"""
__all__ = ["binding", "build"]
