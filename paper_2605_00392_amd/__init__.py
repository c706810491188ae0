"""RTPrune batched visual-token reduction for MI355X (gfx950).

``rtprune`` is the thin ctypes binding over the C-ABI HIP library
(``librtprune.so``, built from ``csrc/``); ``synth`` draws the seeded synthetic
workloads.  Importing the package loads nothing native: the library is opened
on first use and its absence is an error, never a fallback.
"""
__all__ = ["rtprune", "synth"]
