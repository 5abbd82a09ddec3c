"""Channel-gated convolution for MI355X (gfx950).

``paper_1805_12549_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; importing it fails loudly if the library has not
been built.  ``paper_1805_12549_amd.workloads`` makes seeded synthetic inputs.
"""
__all__ = ["binding", "workloads"]
