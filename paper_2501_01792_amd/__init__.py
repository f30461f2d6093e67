"""MI355X-native hybrid KV/activation-cache decode step (arXiv 2501.01792, Sec. 4.2.2).

``paper_2501_01792_amd.binding`` is the ctypes binding of the C-ABI library
(hand-written HIP kernels for gfx950); ``paper_2501_01792_amd.synth`` draws the
seeded synthetic OPT-shaped inputs.  Nothing is loaded at package import.
"""
__all__ = ["binding", "synth"]
