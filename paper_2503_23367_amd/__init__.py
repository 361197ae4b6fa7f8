"""MI355X-native pruned VAR decoding step (FastVAR cached token pruning).

The package is a thin ctypes binding (`binding`) over libfastvar.so, whose
kernels are hand-written HIP for gfx950, plus the seeded synthetic input
generators (`synth`).  Importing the package does not load the library;
`binding.lib()` does, and fails loudly if it has not been built.
"""
__all__ = ["binding", "synth"]
