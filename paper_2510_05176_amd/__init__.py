"""PatternKV hot path for MI355X (gfx950): pattern mining, residual quantize-append
and decode attention over the packed cache, as hand-written HIP kernels behind a
C-ABI library.  ``patternkv`` is the binding; ``synth`` the seeded input generators.

Importing the package does not load the HIP library; ``patternkv`` does, and
raises if it has not been built (there is no CPU fallback).
"""
__all__ = ["patternkv", "synth"]
