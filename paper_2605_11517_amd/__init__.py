"""gnnmi: partition-wise full-graph GNN layers on MI355X behind a C ABI (``libgnnmi.so``).

The Python layer only marshals arguments; every step of the path runs in the HIP kernels of
the shared library.  There is no CPU fallback: if the library is missing, loading fails.
"""
from .binding import (  # noqa: F401
    GNN_BF16, GNN_F32, GNN_GCN, GNN_PART_LP, GNN_PART_RANDOM, GNN_PART_USER, GNN_SAGE_MEAN,
    KERNEL_CLASSES, GnnError, Context, Session, load_library,
)
