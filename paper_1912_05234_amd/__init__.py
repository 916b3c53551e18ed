"""MI355X (gfx950) implementation of one training step of the CNN of
arXiv 1912.05234, behind a C-ABI library (include/cnn.h).

`paper_1912_05234_amd.binding` holds the thin ctypes layer over the library;
`paper_1912_05234_amd.inputs` the seeded synthetic input generators.
Nothing is loaded at import time; the first use of the binding loads the
built library and raises if it is missing.
"""
__all__ = ["binding", "inputs"]
