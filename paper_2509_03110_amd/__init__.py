"""K-replica LSAM step engine for MI355X: HIP kernels behind a C boundary (include/lsam.h)
and its ctypes binding (paper_2509_03110_amd.lsam)."""
from . import lsam  # noqa: F401
