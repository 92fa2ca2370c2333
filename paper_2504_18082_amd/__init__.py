"""COMM-RAND hot path for MI355X (gfx950): thin Python binding over libcommrand.so.

The binding (``paper_2504_18082_amd.binding``) only marshals arguments; every
step of the path runs in the HIP kernels of ``csrc/``.  ``synth`` holds the
seeded input generators.  Nothing is loaded at import time.
"""
__all__ = ["binding", "synth"]
