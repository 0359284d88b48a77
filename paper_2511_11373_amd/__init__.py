"""Routed-expert MoE FFN block for gfx950: Python binding over the C-ABI library.

Importing the package loads nothing native; the shared library is opened on the
first call into `paper_2511_11373_amd.moe` (and that fails loudly if it has
not been built).
"""
