"""Absorbed multi-head latent attention decode for MI355X (gfx950).

``paper_2502_07864_amd.mla`` is the Python binding of the C-ABI library
(hand-written HIP kernels), ``paper_2502_07864_amd.convert`` that of the offline
conversion.  Importing the package itself loads neither torch nor the native
library.
"""
__all__ = ["mla", "convert"]
