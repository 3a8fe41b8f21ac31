"""Data-tiered mini-batch sampling and feature gather for MI355X (gfx950).

``tier``  -- thin ctypes binding of the C-ABI library built from ``csrc/``.
``synth`` -- seeded synthetic inputs (shared with the tests' CPU oracle).
"""
