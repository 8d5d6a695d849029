"""MI355X-native block-masked cross-attention of Beagle's draft decoder.

`synth` draws seeded inputs (NumPy only); `binding` is the ctypes layer over
the C-ABI library built from `csrc/`.  Importing the package loads nothing
native; the library is opened on first use and its absence is an error.
"""
__all__ = ["synth", "binding"]
