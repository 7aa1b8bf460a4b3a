"""CSD verification for MI355X: thin Python binding over the C-ABI HIP library (libcsd.so).

Importing the package is cheap and loads nothing; `paper_2604_13634_amd.binding` loads the
library on first use and raises if it has not been built (there is no fallback path).
"""
__all__ = ["binding", "build"]
