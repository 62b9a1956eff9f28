"""MI355X-native forward/backward of packed variable-length transformer blocks.

``synth`` draws seeded inputs; ``binding`` is the thin ctypes layer over the
C-ABI library built from ``csrc/`` (loaded on first use, never at import).
"""
