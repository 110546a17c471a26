"""ORACLE -- test infrastructure only (never imported by the product path).

Serial CPU evaluation, in double, of the sparse-times-dense product that the
paper's Listing 1 (Section 3.1) defines, plus the parity metric built on it.
"""
