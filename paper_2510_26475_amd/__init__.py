"""MI355X-native speculative-decoding verify step (attention + rejection sampling).

``binding`` wraps the C-ABI library ``librespec.so`` (hand-written HIP for gfx950);
``synth`` draws the seeded synthetic workloads.  Importing the package loads nothing
native; the library is loaded on the first call and its absence is an error.
"""
__all__ = ["binding", "synth"]
