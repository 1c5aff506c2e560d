"""naut-attn: fused attention forward for MI355X (gfx950).

``paper_2604_14825_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; ``paper_2604_14825_amd.synth`` makes the seeded
synthetic inputs.  Nothing here falls back to a CPU implementation.
"""
__version__ = "0.1.0"
