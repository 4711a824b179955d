"""MI355X-native masked attention for Attention Pruning (AP).

The package holds the HIP kernels and their C-ABI library (``csrc/``, declared in
``include/ap.h``), a thin ctypes binding with the same names (``binding``), and the seeded
synthetic input generators (``synth``).  Importing the package does not load the library;
the first call into ``binding`` does, and fails loudly if it has not been built.
"""
__all__ = ["binding", "synth", "build"]
