"""MI355X-native PRESERVE decode step: HIP kernels behind a C-ABI library plus a thin binding.

Importing the package loads nothing; `paper_2501_08192_amd.binding` loads the built library and
fails loudly when it is missing.
"""
__all__ = ["synth", "binding"]
