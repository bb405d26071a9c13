"""DEER hot path for one MI355X: a thin Python binding over the C-ABI HIP library.

Importing the package does not load the library; ``paper_2309_12252_amd.deer`` does,
and fails loudly if it has not been built.
"""
__all__ = ["inputs"]
