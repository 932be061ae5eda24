"""MI355X-native convolutional-layer hot path of ZNN (arXiv 1510.06706).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind a C ABI,
declared in ``include/znn.h``); ``binding`` is the thin ctypes layer with the
same names.  Importing the package does not load the library; the first call
does, and raises if the library has not been built.
"""
__all__ = ["binding", "synth"]
