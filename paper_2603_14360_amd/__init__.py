"""MI355X-native M2RNN recurrent scan (forward + BPTT backward).

The product is the C-ABI library built from ``csrc/`` (hand-written HIP for
gfx950); ``binding`` is a thin ctypes layer over it with the same entry-point
names.  Importing this package loads nothing: the library is opened on first
use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "synth_inputs"]
