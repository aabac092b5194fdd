"""Fused lm_head projection + cross-entropy for MI355X (gfx950).

The compute lives in a C-ABI shared library built from ``csrc/`` (see
``include/flce.h``); ``paper_2511_17599_amd.binding`` is the thin Python
layer over it.  Importing this package loads nothing native: the library is
opened on first use and a missing library is an error, never a fallback.
"""
__all__ = ["inputs"]
