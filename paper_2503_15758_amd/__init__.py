"""MI355X-native tile kernels and AttnFix for Attention2D (arXiv 2503.15758).

The GPU entry points live in `paper_2503_15758_amd.binding` (a ctypes view of
the C-ABI library built from `csrc/`); `synth` holds the seeded input recipe.
Importing the package does not load the library; calling an op does, and fails
loudly if it has not been built.
"""
__all__ = ["binding", "synth"]
