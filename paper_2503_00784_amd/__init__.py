"""MI355X-native verify step of DuoDecoding (arxiv 2503.00784): HIP kernels behind a C ABI.

Importing the package is cheap and loads nothing native; `paper_2503_00784_amd.binding`
loads the shared library and fails loudly if it has not been built.
"""
__all__ = ["inputs", "binding", "build"]
