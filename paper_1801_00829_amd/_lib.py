"""Loads libfuse.so with ctypes and declares the C ABI of include/fuse.h."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfuse.so")

MAX_SIDES = 8


class Dense(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64)]


class CsrDesc(ctypes.Structure):
    _fields_ = [("vals", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("rowptr", ctypes.c_void_p),
                ("rowptr_is64", ctypes.c_int32), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("nnz", ctypes.c_int64)]


class Side(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("m", Dense), ("scalar", ctypes.c_double),
                ("sp", ctypes.POINTER(CsrDesc))]


class Tok(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("arg", ctypes.c_int32), ("imm", ctypes.c_double)]


class Expr(ctypes.Structure):
    _fields_ = [("toks", ctypes.POINTER(Tok)), ("ntoks", ctypes.c_int32)]


_lib = None


def load():
    """Returns the loaded library; raises if libfuse.so has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfuse.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_1801_00829_amd/build.py) first")
    # Share the HIP runtime that PyTorch has loaded: device pointers and streams
    # are only meaningful inside one runtime instance.  Loading torch's copies of
    # the runtime and of hipRTC first makes libfuse's NEEDED entries resolve to them.
    import torch
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib")
    for name in ("libamdhip64.so", "libhiprtc.so"):
        p = os.path.join(tlib, name)
        if os.path.exists(p):
            ctypes.CDLL(p, mode=ctypes.RTLD_GLOBAL)
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    vp, ci, i64p, dp = ctypes.c_void_p, ctypes.c_int, P(ctypes.c_int64), P(ctypes.c_double)
    lib.fuse_cell.argtypes = [P(Expr), P(Dense), P(Side), ci, ci, vp, vp]
    lib.fuse_magg.argtypes = [P(Expr), ci, P(Dense), P(Side), ci, vp, vp]
    lib.fuse_magg_noalloc.argtypes = [P(Expr), ci, P(Dense), P(Side), ci, vp, vp]
    lib.fuse_row.argtypes = [P(Expr), P(Dense), P(CsrDesc), P(Side), ci, ci, vp, vp]
    lib.fuse_outer.argtypes = [P(Expr), P(CsrDesc), P(Dense), P(Dense), P(Side), ci, ci, vp, vp]
    lib.fuse_cell_csr.argtypes = [P(Expr), P(CsrDesc), P(Side), ci, ci, vp, vp]
    lib.fuse_magg_csr.argtypes = [P(Expr), ci, P(CsrDesc), P(Side), ci, vp, vp]
    lib.fuse_prepare_cell_csr.argtypes = [P(Expr), P(CsrDesc), P(Side), ci, ci]
    lib.fuse_prepare_magg_csr.argtypes = [P(Expr), ci, P(CsrDesc), P(Side), ci]
    lib.fuse_prepare_cell.argtypes = [P(Expr), P(Dense), P(Side), ci, ci]
    lib.fuse_prepare_magg.argtypes = [P(Expr), ci, P(Dense), P(Side), ci]
    lib.fuse_prepare_row.argtypes = [P(Expr), P(Dense), P(CsrDesc), P(Side), ci, ci]
    lib.fuse_prepare_outer.argtypes = [P(Expr), P(CsrDesc), P(Dense), P(Dense), P(Side), ci, ci]
    lib.fuse_outer_left_pattern_bytes.argtypes = [P(CsrDesc)]
    lib.fuse_outer_left_pattern_bytes.restype = ctypes.c_size_t
    lib.fuse_outer_left_prepare.argtypes = [P(CsrDesc), vp, vp]
    lib.fuse_outer_left_prepare.restype = ci
    lib.fuse_outer_left_values.argtypes = [P(CsrDesc), vp, vp]
    lib.fuse_outer_left_values.restype = ci
    lib.fuse_outer_left.argtypes = [P(Expr), P(CsrDesc), vp, P(Dense), P(Dense), P(Side), ci, vp, vp]
    lib.fuse_outer_left.restype = ci
    lib.fuse_row_out_count.argtypes = [P(Expr), P(Dense), P(CsrDesc), P(Side), ci, ci, i64p]
    lib.fuse_row_out_count.restype = ci
    lib.fuse_check_csr.argtypes = [P(CsrDesc), vp]
    for f in (lib.fuse_check_csr, lib.fuse_cell_csr, lib.fuse_magg_csr, lib.fuse_prepare_cell_csr, lib.fuse_prepare_magg_csr,
              lib.fuse_cell, lib.fuse_magg, lib.fuse_magg_noalloc, lib.fuse_row, lib.fuse_outer, lib.fuse_prepare_cell,
              lib.fuse_prepare_magg, lib.fuse_prepare_row, lib.fuse_prepare_outer):
        f.restype = ci
    lib.fuse_last_error.restype = ctypes.c_char_p
    lib.fuse_last_kernel.restype = ctypes.c_char_p
    lib.fuse_cache_stats.argtypes = [i64p, i64p, dp]
    lib.fuse_cache_stats.restype = ci
    lib.fuse_cache_clear.restype = None
    lib.fuse_cache_disk_hits.argtypes = []
    lib.fuse_cache_disk_hits.restype = ctypes.c_int64
    lib.fuse_last_source.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    lib.fuse_last_source.restype = ctypes.c_size_t
    lib.fuse_probe_copy.argtypes = [vp, vp, ctypes.c_int64, ci, vp]
    lib.fuse_probe_copy.restype = ci
    lib.fuse_probe_read.argtypes = [vp, ctypes.c_int64, ci, vp, vp]
    lib.fuse_probe_read.restype = ci
    lib.fuse_probe_gather.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_int64, ci, vp, vp]
    lib.fuse_probe_gather.restype = ci
    _lib = lib
    return lib
