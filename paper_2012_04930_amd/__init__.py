"""gcn355: full-batch Kipf-Welling GCN training step on one partition, HIP kernels for MI355X.

`from paper_2012_04930_amd import binding` gives the ctypes face of libgcn355.so; the functions
there have the names of the C entry points declared in include/gcn355.h.
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
