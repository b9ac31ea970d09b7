"""FusedMM (fused SDDMM-SpMM) for AMD MI355X (gfx950).

``paper_2011_06391_amd.binding`` is the thin ctypes layer over the C-ABI
library ``libfusedmm.so`` (hand-written HIP kernels); ``synth`` holds the
seeded input generators; ``model`` the byte/flop model of the kernel.
Nothing is imported eagerly so that host-only tools (generators, the model)
work without a GPU.
"""

__all__ = ["binding", "synth", "model", "build"]
