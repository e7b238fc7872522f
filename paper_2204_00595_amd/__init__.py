"""MI355X-native Monarch multiply (y = x M^T, M = P L P^T R), forward and backward.

The work is done by hand-written HIP kernels behind a C-ABI shared library
(``include/monarch.h``); this package is the thin Python binding over it plus
the seeded synthetic-input generator used by tests and benchmarks.
"""
__all__ = ["synth"]
