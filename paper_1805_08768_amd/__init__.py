"""MI355X-native Sparse Binary Compression (arXiv 1805.08768).

`synth` holds the seeded input generators (NumPy only).  `binding` is the thin
ctypes layer over the C-ABI library `libsbc.so` built from `csrc/`; it is
imported on demand so that shape and generator helpers work without a GPU.
"""

__all__ = ["synth", "binding"]
