"""MI355X-native shifted-window attention (AERIS hot path).

``binding`` wraps the C-ABI library built from ``csrc/``; ``synth`` holds the
seeded input recipes.  Importing the package loads no native code; the first
call into ``binding`` does, and raises if the library has not been built.
"""
__all__ = ["binding", "synth"]
