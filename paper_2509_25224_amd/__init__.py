"""Absorbed-MLA decode attention for MI355X (gfx950) with the exponent-add rescale.

`amla` holds the ctypes binding of the C-ABI library; `workloads` the seeded synthetic
inputs; `accounting` the FLOP/byte formulas.  Importing the package does not load the
native library; `paper_2509_25224_amd.amla` does, and raises if it has not been built.
"""
