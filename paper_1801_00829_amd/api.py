"""Thin wrappers with the names of the C entry points (argument marshalling only)."""
import ctypes
from collections import namedtuple

from . import _lib as L

AGG = {"none": 0, "full": 1, "row": 2, "col": 3, "col_t": 4, "right_mm": 5, "left_mm": 6}
SIDE = {"matrix": 0, "colvec": 1, "rowvec": 2, "scalar": 3, "rhs": 4, "kvec": 5, "sparse": 6}
OPS = {
    "main": 1, "side": 2, "const": 3, "uvdot": 4,
    "neg": 16, "abs": 17, "sqrt": 18, "exp": 19, "log": 20, "pow2": 21, "sign": 22, "neq0": 23,
    "sigmoid": 24,
    "add": 32, "sub": 33, "mul": 34, "div": 35, "min": 36, "max": 37, "pow": 38,
    "lt": 39, "le": 40, "gt": 41, "ge": 42, "eq": 43, "ne": 44,
    "rowsum": 48, "dot": 49, "matmult": 50, "outerk": 51,
}

Csr = namedtuple("Csr", "rowptr colidx vals shape")
"""CSR matrix on the device: rowptr (int32 or int64, m+1), colidx (int32), vals (float64), (m, n)."""


class FuseError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libfuse error %d: %s" % (code, msg))
        self.code = code


def lib_path():
    return L.LIB_PATH


def _check(rc):
    if rc != 0:
        raise FuseError(rc, L.load().fuse_last_error().decode("utf-8", "replace"))


_EXPR_CACHE = {}


def _expr(tokens):
    """Symbolic postfix list, e.g. [("main",), ("side", 0), ("mul",)] -> (Expr, keep-alive).
    Marshalled descriptors are kept by value of the list, so a loop that issues the same
    operator again does not rebuild the token array."""
    try:
        key = tuple(tuple(t) for t in tokens)
        hit = _EXPR_CACHE.get(key)
    except TypeError:                      # unhashable token entries: marshal without caching
        key, hit = None, None
    if hit is not None:
        return hit
    arr = (L.Tok * max(len(tokens), 1))()
    for i, t in enumerate(tokens):
        name = t[0]
        if name not in OPS:
            raise ValueError("unknown token %r" % (t,))
        arr[i].op = OPS[name]
        arr[i].arg = int(t[1]) if name == "side" else 0
        arr[i].imm = float(t[1]) if name == "const" else 0.0
    res = (L.Expr(arr, len(tokens)), arr)
    if key is not None:
        if len(_EXPR_CACHE) > 1024:
            _EXPR_CACHE.clear()
        _EXPR_CACHE[key] = res
    return res


def _on_gpu(t, what):
    """Kernels dereference the pointer on the device: a host tensor would fault the GPU, not raise."""
    if not t.is_cuda:
        raise ValueError("%s must be a CUDA (HIP) tensor, got device %s" % (what, t.device))
    return t


def _dense(t, rows=None, cols=None):
    """2-D (or 1-D) float64 tensor with unit column stride -> Dense descriptor."""
    import torch
    if t is None:
        return None
    if isinstance(t, tuple):                      # shape only (prepare_*): (rows, cols[, ld])
        r, c = int(t[0]), int(t[1])
        return L.Dense(None, r, c, int(t[2]) if len(t) > 2 else max(c, 1))
    if t.dtype != torch.float64:
        raise TypeError("libfuse matrices are float64")
    _on_gpu(t, "matrix")
    if t.dim() == 1:
        t = t.view(-1, 1) if cols == 1 else t.view(1, -1)
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("need a 2-D tensor with unit column stride")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    if t.shape[1] == 1 and t.shape[0] > 1:
        ld = t.stride(0)
    return L.Dense(t.data_ptr(), t.shape[0], t.shape[1], max(int(ld), 1))


def _sides(sides, m, n):
    """[(kind, tensor | float | shape-tuple)] -> (Side array, count)."""
    import torch
    arr = (L.Side * max(len(sides), 1))()
    arr._keep = []                                        # CSR descriptors of sparse sides live as long as the array
    for k, (kind, val) in enumerate(sides):
        arr[k].kind = SIDE[kind]
        if kind == "scalar":
            arr[k].scalar = float(val)
        elif kind == "sparse":                            # a Csr of device tensors, or prepare_*: (is64, None, nnz, shape)
            desc = _csr(val)
            arr._keep.append(desc)
            arr[k].sp = ctypes.pointer(desc)
        elif kind in ("rhs", "kvec"):
            if isinstance(val, tuple):                    # shape only: (rows, k)
                arr[k].m = L.Dense(None, int(val[0]), int(val[1]), int(val[1]))
            else:
                arr[k].m = _dense(val)
        elif kind == "colvec":
            if isinstance(val, tuple) or val is None:
                arr[k].m = L.Dense(None, m, 1, 1)
            else:
                v = val.view(-1, 1) if val.dim() == 1 else val
                if v.dtype != torch.float64:
                    raise TypeError("libfuse vectors are float64")
                _on_gpu(v, "column-vector side")
                arr[k].m = L.Dense(v.data_ptr(), v.shape[0], 1, max(int(v.stride(0)), 1))
        elif kind == "rowvec":
            if isinstance(val, tuple) or val is None:
                arr[k].m = L.Dense(None, 1, n, max(n, 1))
            else:
                v = val.reshape(1, -1) if val.dim() == 1 else val
                if v.dtype != torch.float64:
                    raise TypeError("libfuse vectors are float64")
                _on_gpu(v, "row-vector side")
                if v.shape[0] != 1 and v.shape[1] == 1:      # an n x 1 column used by column index
                    if v.stride(0) != 1:
                        raise ValueError("row-vector side must be contiguous")
                    v = v.view(1, -1)
                if v.shape[1] > 1 and v.stride(1) != 1:
                    raise ValueError("row-vector side must be contiguous")
                arr[k].m = L.Dense(v.data_ptr(), 1, v.shape[1], max(v.shape[1], 1))
        else:
            arr[k].m = _dense(val if val is not None else (m, n))
    return arr, len(sides)


def _csr(x):
    import torch
    rowptr, colidx, vals, shape = x
    m, n = int(shape[0]), int(shape[1])
    if isinstance(rowptr, int):                   # prepare_*: (is64, None, nnz, shape)
        return L.CsrDesc(None, None, None, int(rowptr), m, n, int(vals))
    if colidx.dtype != torch.int32 or vals.dtype != torch.float64:
        raise TypeError("CSR needs int32 column indices and float64 values")
    for t_, what in ((rowptr, "CSR row offsets"), (colidx, "CSR column indices"), (vals, "CSR values")):
        _on_gpu(t_, what)
    if rowptr.dtype not in (torch.int32, torch.int64):
        raise TypeError("CSR row offsets must be int32 or int64")
    if not (rowptr.is_contiguous() and colidx.is_contiguous() and vals.is_contiguous()):
        raise ValueError("CSR arrays must be contiguous")
    if rowptr.numel() != m + 1 or colidx.numel() != vals.numel():
        raise ValueError("CSR array lengths do not match the shape")
    return L.CsrDesc(vals.data_ptr(), colidx.data_ptr(), rowptr.data_ptr(),
                     1 if rowptr.dtype == torch.int64 else 0, m, n, vals.numel())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _out(out, count, like):
    import torch
    if out is None:
        out = torch.empty(int(count), dtype=torch.float64, device=like.device)
    elif out.dtype != torch.float64 or not out.is_contiguous() or out.numel() < count or not out.is_cuda:
        raise ValueError("out must be a contiguous float64 CUDA tensor with at least %d elements" % count)
    return out


def _agg_count(agg, m, n, vec_result=True, nnz=None):
    if agg == "full":
        return 1
    if agg == "row":
        return m
    if agg in ("col", "col_t"):
        return n
    if nnz is not None and vec_result:
        return nnz
    return m * n if vec_result else m


# --------------------------------------------------------------------- entry points ---

def fuse_cell(expr, X, sides=(), agg="full", out=None, stream=None):
    """C: fuse_cell.  X: cuda float64 (m, n).  Returns the out tensor (flat)."""
    lib = L.load()
    e, keep = _expr(expr)
    xd = _dense(X)
    sa, ns = _sides(list(sides), xd.rows, xd.cols)
    out = _out(out, _agg_count(agg, xd.rows, xd.cols), X)
    _check(lib.fuse_cell(ctypes.byref(e), ctypes.byref(xd), sa, ns, AGG[agg], out.data_ptr(), _stream(stream)))
    return out


def fuse_magg(exprs, X, sides=(), out=None, stream=None):
    """C: fuse_magg.  k full aggregates in one scan; returns k values."""
    lib = L.load()
    pairs = [_expr(e) for e in exprs]
    ea = (L.Expr * len(pairs))(*[p[0] for p in pairs])
    xd = _dense(X)
    sa, ns = _sides(list(sides), xd.rows, xd.cols)
    out = _out(out, len(pairs), X)
    _check(lib.fuse_magg(ea, len(pairs), ctypes.byref(xd), sa, ns, out.data_ptr(), _stream(stream)))
    return out


def fuse_magg_noalloc(exprs, X, sides, out, stream=None):
    """C: fuse_magg_noalloc.  The caller brings `out` (k float64 values on the device): nothing is allocated."""
    lib = L.load()
    pairs = [_expr(e) for e in exprs]
    ea = (L.Expr * len(pairs))(*[p[0] for p in pairs])
    xd = _dense(X)
    sa, ns = _sides(list(sides), xd.rows, xd.cols)
    if out is None:
        raise ValueError("fuse_magg_noalloc needs the caller's output tensor")
    out = _out(out, len(pairs), X)
    _check(lib.fuse_magg_noalloc(ea, len(pairs), ctypes.byref(xd), sa, ns, out.data_ptr(), _stream(stream)))
    return out


def fuse_cell_csr(expr, X, sides=(), agg="full", out=None, stream=None):
    """C: fuse_cell_csr.  X: Csr of device tensors; sparse-safe Cell body at the stored cells."""
    lib = L.load()
    e, keep = _expr(expr)
    xs = _csr(X)
    sa, ns = _sides(list(sides), xs.rows, xs.cols)
    out = _out(out, _agg_count(agg, xs.rows, xs.cols, True, nnz=xs.nnz), X.vals)
    _check(lib.fuse_cell_csr(ctypes.byref(e), ctypes.byref(xs), sa, ns, AGG[agg], out.data_ptr(), _stream(stream)))
    return out


def fuse_magg_csr(exprs, X, sides=(), out=None, stream=None):
    """C: fuse_magg_csr.  k full aggregates over the stored cells of X in one scan."""
    lib = L.load()
    pairs = [_expr(e) for e in exprs]
    ea = (L.Expr * len(pairs))(*[p[0] for p in pairs])
    xs = _csr(X)
    sa, ns = _sides(list(sides), xs.rows, xs.cols)
    out = _out(out, len(pairs), X.vals)
    _check(lib.fuse_magg_csr(ea, len(pairs), ctypes.byref(xs), sa, ns, out.data_ptr(), _stream(stream)))
    return out


def prepare_cell_csr(expr, shape, nnz, sides=(), agg="full", rowptr64=False):
    lib = L.load()
    e, keep = _expr(expr)
    xs = L.CsrDesc(None, None, None, int(rowptr64), shape[0], shape[1], int(nnz))
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    _check(lib.fuse_prepare_cell_csr(ctypes.byref(e), ctypes.byref(xs), sa, ns, AGG[agg]))


def prepare_magg_csr(exprs, shape, nnz, sides=(), rowptr64=False):
    lib = L.load()
    pairs = [_expr(e) for e in exprs]
    ea = (L.Expr * len(pairs))(*[p[0] for p in pairs])
    xs = L.CsrDesc(None, None, None, int(rowptr64), shape[0], shape[1], int(nnz))
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    _check(lib.fuse_prepare_magg_csr(ea, len(pairs), ctypes.byref(xs), sa, ns))


def _row_out_count(lib, e, xd, xs, sa, ns, agg):
    """C: fuse_row_out_count -- the library says how many values the result has."""
    cnt = ctypes.c_int64()
    _check(lib.fuse_row_out_count(ctypes.byref(e), ctypes.byref(xd) if xd is not None else None,
                                  ctypes.byref(xs) if xs is not None else None, sa, ns, AGG[agg], ctypes.byref(cnt)))
    return cnt.value


def fuse_row(expr, X, sides=(), agg="col_t", out=None, stream=None):
    """C: fuse_row.  X: cuda float64 (m, n) tensor or a Csr of device tensors."""
    lib = L.load()
    e, keep = _expr(expr)
    sides = list(sides)
    if isinstance(X, Csr):
        xs = _csr(X)
        m, n = xs.rows, xs.cols
        sa, ns = _sides(sides, m, n)
        out = _out(out, _row_out_count(lib, e, None, xs, sa, ns, agg), X.vals)
        _check(lib.fuse_row(ctypes.byref(e), None, ctypes.byref(xs), sa, ns, AGG[agg], out.data_ptr(),
                            _stream(stream)))
    else:
        xd = _dense(X)
        sa, ns = _sides(sides, xd.rows, xd.cols)
        out = _out(out, _row_out_count(lib, e, xd, None, sa, ns, agg), X)
        _check(lib.fuse_row(ctypes.byref(e), ctypes.byref(xd), None, sa, ns, AGG[agg], out.data_ptr(),
                            _stream(stream)))
    return out


def fuse_outer(expr, X, U, V, sides=(), agg="full", out=None, stream=None):
    """C: fuse_outer.  X: Csr of device tensors; U (m, r), V (n, r) cuda float64."""
    lib = L.load()
    e, keep = _expr(expr)
    xs = _csr(X)
    ud, vd = _dense(U), _dense(V)
    sa, ns = _sides(list(sides), xs.rows, xs.cols)
    count = {"full": 1, "none": xs.nnz, "right_mm": xs.rows * ud.cols, "left_mm": xs.cols * ud.cols}[agg]
    out = _out(out, count, X.vals)
    _check(lib.fuse_outer(ctypes.byref(e), ctypes.byref(xs), ctypes.byref(ud), ctypes.byref(vd), sa, ns,
                          AGG[agg], out.data_ptr(), _stream(stream)))
    return out


def outer_left_prepare(X, stream=None):
    """C: fuse_outer_left_pattern_bytes + fuse_outer_left_prepare.  Returns the prepared pattern of X (a uint8
    device tensor that the caller keeps for as long as it calls fuse_outer_left with it)."""
    import torch
    lib = L.load()
    xs = _csr(X)
    nbytes = int(lib.fuse_outer_left_pattern_bytes(ctypes.byref(xs)))
    pattern = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=X.vals.device)
    _check(lib.fuse_outer_left_prepare(ctypes.byref(xs), pattern.data_ptr(), _stream(stream)))
    return pattern


def outer_left_values(X, pattern, stream=None):
    """C: fuse_outer_left_values.  X has new values on the same structure: refresh the pattern's copy."""
    xs = _csr(X)
    _on_gpu(pattern, "pattern")
    _check(L.load().fuse_outer_left_values(ctypes.byref(xs), pattern.data_ptr(), _stream(stream)))


def fuse_outer_left(expr, X, pattern, U, V, sides=(), out=None, stream=None):
    """C: fuse_outer_left.  left_mm over a pattern from outer_left_prepare (values as of the last prepare /
    outer_left_values call)."""
    lib = L.load()
    e, keep = _expr(expr)
    xs = _csr(X)
    ud, vd = _dense(U), _dense(V)
    sa, ns = _sides(list(sides), xs.rows, xs.cols)
    out = _out(out, xs.cols * ud.cols, X.vals)
    _on_gpu(pattern, "pattern")
    _check(lib.fuse_outer_left(ctypes.byref(e), ctypes.byref(xs), pattern.data_ptr(), ctypes.byref(ud), ctypes.byref(vd),
                               sa, ns, out.data_ptr(), _stream(stream)))
    return out


def check_csr(X, stream=None):
    """C: fuse_check_csr.  Raises FuseError (FUSE_ESHAPE) if the CSR structure is malformed; waits for the stream."""
    lib = L.load()
    xs = _csr(X)
    _check(lib.fuse_check_csr(ctypes.byref(xs), _stream(stream)))


# ----------------------------------------------------- compile-only (no device needed) ---

def prepare_cell(expr, shape, sides=(), agg="full", ld=None):
    """C: fuse_prepare_cell.  shape = (m, n); sides = [(kind, None | float)]."""
    lib = L.load()
    e, keep = _expr(expr)
    xd = L.Dense(None, shape[0], shape[1], ld or max(shape[1], 1))
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    _check(lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(xd), sa, ns, AGG[agg]))


def prepare_magg(exprs, shape, sides=()):
    lib = L.load()
    pairs = [_expr(e) for e in exprs]
    ea = (L.Expr * len(pairs))(*[p[0] for p in pairs])
    xd = L.Dense(None, shape[0], shape[1], max(shape[1], 1))
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    _check(lib.fuse_prepare_magg(ea, len(pairs), ctypes.byref(xd), sa, ns))


def prepare_row(expr, shape, sides=(), agg="col_t", nnz=None, rowptr64=False):
    """C: fuse_prepare_row.  nnz=None: dense main input; else CSR with that many stored cells."""
    lib = L.load()
    e, keep = _expr(expr)
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    if nnz is None:
        xd = L.Dense(None, shape[0], shape[1], max(shape[1], 1))
        _check(lib.fuse_prepare_row(ctypes.byref(e), ctypes.byref(xd), None, sa, ns, AGG[agg]))
    else:
        xs = L.CsrDesc(None, None, None, int(rowptr64), shape[0], shape[1], int(nnz))
        _check(lib.fuse_prepare_row(ctypes.byref(e), None, ctypes.byref(xs), sa, ns, AGG[agg]))


def prepare_outer(expr, shape, rank, nnz, sides=(), agg="full", rowptr64=False):
    lib = L.load()
    e, keep = _expr(expr)
    xs = L.CsrDesc(None, None, None, int(rowptr64), shape[0], shape[1], int(nnz))
    ud = L.Dense(None, shape[0], rank, rank)
    vd = L.Dense(None, shape[1], rank, rank)
    sa, ns = _sides([(k, v) for k, v in sides], shape[0], shape[1])
    _check(lib.fuse_prepare_outer(ctypes.byref(e), ctypes.byref(xs), ctypes.byref(ud), ctypes.byref(vd), sa, ns,
                                  AGG[agg]))


# ------------------------------------------------------------------------- utilities ---

def cache_stats():
    """(hits, misses, compile_ms) of the plan cache."""
    h, m, ms = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_double()
    L.load().fuse_cache_stats(ctypes.byref(h), ctypes.byref(m), ctypes.byref(ms))
    return h.value, m.value, ms.value


def cache_clear():
    L.load().fuse_cache_clear()


def cache_disk_hits():
    """Plan-cache misses served from FUSE_CACHE_DIR since load / last clear."""
    return int(L.load().fuse_cache_disk_hits())


def last_source():
    lib = L.load()
    n = lib.fuse_last_source(None, 0)
    buf = ctypes.create_string_buffer(n + 1)
    lib.fuse_last_source(buf, n + 1)
    return buf.value.decode()


def last_kernel():
    return L.load().fuse_last_kernel().decode()


def probe_copy(dst, src, blocks, stream=None):
    _check(L.load().fuse_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(), int(blocks), _stream(stream)))


def probe_read(src, sink, blocks, stream=None, n_doubles=None):
    """C: fuse_probe_read over the first n_doubles values of src (default all; 0: a kernel that reads nothing)."""
    n = src.numel() if n_doubles is None else int(n_doubles)
    if n < 0 or n > src.numel():
        raise ValueError("n_doubles out of range")
    _check(L.load().fuse_probe_read(src.data_ptr(), n, int(blocks), sink.data_ptr(), _stream(stream)))


def probe_gather(table, idx, sink, blocks, stream=None):
    """C: fuse_probe_gather.  table: cuda float64 (rows, row_doubles); idx: cuda int32 row numbers."""
    import torch
    if table.dtype != torch.float64 or idx.dtype != torch.int32 or table.dim() != 2 or table.stride(1) != 1:
        raise TypeError("probe_gather needs a float64 table with unit column stride and int32 indices")
    for t_, what in ((table, "table"), (idx, "idx"), (sink, "sink")):
        _on_gpu(t_, what)
    if not idx.is_contiguous():
        raise ValueError("idx must be contiguous")
    _check(L.load().fuse_probe_gather(table.data_ptr(), table.shape[0], table.shape[1], table.stride(0),
                                      idx.data_ptr(), idx.numel(), int(blocks), sink.data_ptr(), _stream(stream)))
