"""MI355X-native forward path of STILL's intra-layer hybrid attention.

`synth` holds the seeded input generators; `binding` the ctypes wrapper around the
C-ABI library built from `csrc/` (loaded lazily, so importing the package never
needs a GPU or a built library).
"""
__all__ = ["synth", "binding", "build"]
