"""MI355X-native kernels for the pruned-prefill hot path of ViTCoP (arXiv 2601.17818).

The work is done by libvitcop.so (hand-written HIP for gfx950, C ABI declared in
include/vitcop.h).  ``binding`` is a thin ctypes layer with the same names; it
marshals arguments only.  There is no CPU fallback: importing ``binding``
fails if the library has not been built (``python -m paper_2601_17818_amd.build``).
"""
