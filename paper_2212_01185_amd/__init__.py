"""Per-pixel causal-context lossless image coding on MI355X (gfx950).

``synth`` holds the seeded input generators; ``binding`` is the thin ctypes
layer over the C-ABI library built from ``csrc/``.  Importing the package
loads nothing native; the library is opened on first use and raises if absent.
"""
