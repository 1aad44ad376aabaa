"""Python binding of libfuse: fused-operator templates (Cell, MAgg, Row, Outer) on MI355X.

Only argument marshalling happens here; every step of a call runs in the HIP
kernels of ``libfuse.so`` (see ``include/fuse.h``).  PyTorch is used for device
memory and streams.
"""
from .api import (FuseError, Csr, fuse_cell, fuse_magg, fuse_magg_noalloc, fuse_row, fuse_outer,  # noqa: F401
                  fuse_cell_csr, fuse_magg_csr, check_csr, outer_left_prepare, outer_left_values, fuse_outer_left, prepare_cell_csr, prepare_magg_csr,
                  prepare_cell, prepare_magg, prepare_row, prepare_outer,
                  cache_stats, cache_clear, cache_disk_hits, last_source, last_kernel, probe_copy, probe_read, probe_gather,
                  AGG, SIDE, OPS, lib_path)
