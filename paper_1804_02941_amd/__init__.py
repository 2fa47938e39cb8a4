"""MI355X-native hot path of distribution-aware binarization (arXiv 1804.02941).

The package holds the HIP sources of the C-ABI library (``csrc/``), the build
step (``build``), the thin ctypes binding (``binding``) and the seeded input
generators (``workloads``).  Importing the package loads nothing; the shared
library is opened on the first call into ``binding``.
"""
