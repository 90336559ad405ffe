"""MI355X-native 2D stencil skeleton with workgroup-size sweep (libstencil).

Importing the package loads nothing native; `paper_1511_02490_amd.libstencil` is the
thin binding over the C-ABI library and fails loudly if that library is not built.
"""

__all__ = ["workloads", "libstencil"]
