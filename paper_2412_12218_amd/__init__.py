"""Sparse neighbour aggregation for GCN / AGNN on AMD MI355X (gfx950), after FTC-GNN.

The product is the C-ABI library libftc.so (see include/ftc.h); `binding` is a thin ctypes
layer that passes torch device pointers through.  Importing this package does not load
the library; `binding.lib()` does and raises if it has not been built.
"""
from . import binding  # noqa: F401
