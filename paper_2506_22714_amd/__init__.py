"""MI355X-native SpMM / SDDMM with a 2D-aware split between an MFMA dense-tile
path and a VALU scalar path (after arXiv 2506.22714, "Libra").

The work is done by a C-ABI shared library built from ``csrc/`` (see
``include/libra.h``); :mod:`.binding` marshals arguments to it and nothing else.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""

__all__ = ["binding", "workloads"]
