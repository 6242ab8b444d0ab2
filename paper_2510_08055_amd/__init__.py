"""MI355X-native MoE expert-FFN hot path for chunked vs layered prefill.

`paper_2510_08055_amd.binding` is the thin ctypes layer over the C-ABI library
(hand-written HIP kernels for gfx950); `paper_2510_08055_amd.inputs` draws the
seeded synthetic workloads.  Importing the package loads neither.
"""
__all__ = ["binding", "inputs"]
