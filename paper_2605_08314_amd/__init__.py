"""MI355X-native factorized-linear hot path (y = (x U) V) of an SVD-compressed transformer.

``paper_2605_08314_amd.binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/`` (hand-written HIP for gfx950); ``paper_2605_08314_amd.synth`` holds the seeded
synthetic input recipes.  Importing the package does not load the HIP library; importing
``binding`` does, and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
