"""MI355X-native MXFP4 weight-only-quantised linear layer (arXiv 2503.13565, section 3.4.3).

The work is done by hand-written HIP kernels for gfx950 behind a C-ABI shared library
(``include/mxfp4.h``); :mod:`paper_2503_13565_amd.binding` marshals torch tensors into it.
Importing this package does not load the library; the first call does, and fails loudly if
it has not been built.
"""

__all__ = ["binding", "synth"]
