"""MI355X-native DynTS decode hot path: HIP kernels behind a C ABI, with a thin Python binding.

Importing the package loads nothing; `paper_2601_18383_amd.binding` loads the
built library (and fails loudly when it is missing).
"""
__all__ = ["configs", "synth", "binding", "build"]
