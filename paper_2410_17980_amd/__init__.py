"""Causal stick-breaking attention for MI355X (gfx950).

The product is the C-ABI library built from csrc/ (see include/sb_attn.h);
`binding` is the thin ctypes layer over it and `inputs` the seeded input recipes.
Nothing is loaded at import time.
"""
__all__ = ["binding", "inputs", "build"]
