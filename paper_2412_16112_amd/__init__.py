"""MI355X-native CLEAR local attention (arXiv 2412.16112, Sec. 3.2): Python binding of the C-ABI library.

Importing the package loads nothing; `paper_2412_16112_amd.clear_attn` opens the HIP library
(and fails loudly if it has not been built), `paper_2412_16112_amd.inputs` holds the seeded
synthetic-input recipes shared by the tests and the bench.
"""
__all__ = ["clear_attn", "inputs"]
