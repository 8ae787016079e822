"""MI355X-native DAG-structured attention (MedVerse attention, arXiv 2602.07529 section 4.2).

The product is the C-ABI library built from csrc/ (see include/dagattn.h); `binding` is a thin
ctypes layer with the same entry-point names.
"""
from . import binding  # noqa: F401
