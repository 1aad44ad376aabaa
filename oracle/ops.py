"""Basic operators of the unfused plans -- TEST INFRASTRUCTURE ONLY.

Each function is one basic linear-algebra operator as the paper's "Base"
baseline executes it (Sec. 5.1 "Baselines"; Sec. 1 "Fusion Opportunities"):
one pass over the inputs, a freshly allocated output.  Element-wise operators
are numpy's (IEEE fp64, one rounding per element, library ``log``/``exp``);
aggregates and products are the C routines of ``oracle_ops.c`` which accumulate
in extended precision.

CSR matrices are passed as ``Csr`` tuples (rowptr int64[m+1], colidx int32,
vals float64, shape).
"""
import ctypes
from collections import namedtuple

import numpy as np

from . import build as _build

Csr = namedtuple("Csr", "rowptr colidx vals shape")

_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.oracle_sum.restype = ctypes.c_double
        lib.oracle_acc_size.restype = ctypes.c_size_t
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the C operators will use."""
    return int(_c().oracle_threads())


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def _i(x):
    return ctypes.c_int64(int(x))


def _f64(a):
    a = np.asarray(a, dtype=np.float64)
    return a


def _rowmajor(a):
    """2-D float64 array with unit column stride; returns (array, ld)."""
    a = _f64(a)
    assert a.ndim == 2
    if a.strides[1] != 8 or a.strides[0] % 8 or (a.shape[0] > 1 and a.strides[0] < 8 * a.shape[1]):
        a = np.ascontiguousarray(a)
    ld = a.strides[0] // 8 if a.shape[0] > 1 else max(a.shape[1], 1)
    return a, ld


def make_csr(rowptr, colidx, vals, shape) -> Csr:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    m, n = int(shape[0]), int(shape[1])
    assert rowptr.shape == (m + 1,) and rowptr[0] == 0
    assert colidx.shape == vals.shape == (int(rowptr[-1]),)
    return Csr(rowptr, colidx, vals, (m, n))


# ------------------------------------------------------------ element-wise ---

_UNARY = {
    "neg": np.negative,
    "abs": np.abs,
    "sqrt": np.sqrt,
    "exp": np.exp,
    "log": np.log,
    "pow2": lambda a: a * a,
    "sign": np.sign,
    "neq0": lambda a: (a != 0).astype(np.float64),
    "sigmoid": lambda a: 1.0 / (1.0 + np.exp(-a)),
}

_BINARY = {
    "add": np.add,
    "sub": np.subtract,
    "mul": np.multiply,
    "div": np.divide,
    "min": np.minimum,
    "max": np.maximum,
    "pow": np.power,
    "lt": lambda a, b: (a < b).astype(np.float64),
    "le": lambda a, b: (a <= b).astype(np.float64),
    "gt": lambda a, b: (a > b).astype(np.float64),
    "ge": lambda a, b: (a >= b).astype(np.float64),
    "eq": lambda a, b: (a == b).astype(np.float64),
    "ne": lambda a, b: (a != b).astype(np.float64),
}

UNARY_NAMES = tuple(_UNARY)
BINARY_NAMES = tuple(_BINARY)


def ew_unary(op, a):
    """Element-wise unary operator; returns a new array."""
    with np.errstate(all="ignore"):
        return np.array(_UNARY[op](_f64(a)), dtype=np.float64)


def ew_binary(op, a, b):
    """Element-wise binary operator with numpy broadcasting; returns a new array."""
    with np.errstate(all="ignore"):
        return np.array(_BINARY[op](_f64(a), _f64(b)), dtype=np.float64)


# --------------------------------------------------------------- aggregates ---

def sum_full(a) -> float:
    """sum(A) over all cells."""
    a = np.ascontiguousarray(_f64(a)).reshape(-1)
    return float(_c().oracle_sum(_p(a), _i(a.size)))


def row_sums(a):
    """rowSums(A) -> vector of length m."""
    a, ld = _rowmajor(a)
    m, n = a.shape
    out = np.empty(m, dtype=np.float64)
    _c().oracle_row_sums(_p(a), _i(m), _i(n), _i(ld), _p(out))
    return out


def col_sums(a):
    """colSums(A) -> vector of length n."""
    a, ld = _rowmajor(a)
    m, n = a.shape
    out = np.empty(n, dtype=np.float64)
    _c().oracle_col_sums(_p(a), _i(m), _i(n), _i(ld), _p(out))
    return out


# ----------------------------------------------------------------- products ---

def matvec(x, v):
    """X %*% v for dense X (m x n) and a vector v of length n."""
    x, ld = _rowmajor(x)
    m, n = x.shape
    v = np.ascontiguousarray(_f64(v)).reshape(-1)
    assert v.size == n
    q = np.empty(m, dtype=np.float64)
    _c().oracle_matvec(_p(x), _i(m), _i(n), _i(ld), _p(v), _p(q))
    return q


def t_matvec(x, q):
    """t(X) %*% q for dense X (m x n) and a vector q of length m."""
    x, ld = _rowmajor(x)
    m, n = x.shape
    q = np.ascontiguousarray(_f64(q)).reshape(-1)
    assert q.size == m
    out = np.empty(n, dtype=np.float64)
    _c().oracle_t_matvec(_p(x), _i(m), _i(n), _i(ld), _p(q), _p(out))
    return out


def matmul(a, b):
    """A %*% B for dense A (m x n) and B (n x k) -> m x k."""
    a, lda = _rowmajor(a)
    b, ldb = _rowmajor(b)
    assert a.shape[1] == b.shape[0]
    c = np.empty((a.shape[0], b.shape[1]), dtype=np.float64)
    _c().oracle_matmul(_p(a), _i(a.shape[0]), _i(a.shape[1]), _i(lda), _p(b), _i(b.shape[1]), _i(ldb), _p(c))
    return c


def t_matmul(a, q):
    """t(A) %*% Q for dense A (m x n) and Q (m x k) -> n x k."""
    a, lda = _rowmajor(a)
    q, ldq = _rowmajor(q)
    assert a.shape[0] == q.shape[0]
    c = np.empty((a.shape[1], q.shape[1]), dtype=np.float64)
    _c().oracle_t_matmul(_p(a), _i(a.shape[0]), _i(a.shape[1]), _i(lda), _p(q), _i(q.shape[1]), _i(ldq), _p(c))
    return c


def _work(n):
    return np.zeros(int(n) * int(_c().oracle_acc_size()) + 16, dtype=np.uint8)


def csr_matvec(x: Csr, v):
    """X %*% v for CSR X."""
    m, n = x.shape
    v = np.ascontiguousarray(_f64(v)).reshape(-1)
    assert v.size == n
    q = np.empty(m, dtype=np.float64)
    _c().oracle_csr_matvec(_p(x.rowptr), _p(x.colidx), _p(x.vals), _i(m), _p(v), _p(q))
    return q


def csr_t_matvec(x: Csr, q):
    """t(X) %*% q for CSR X."""
    m, n = x.shape
    q = np.ascontiguousarray(_f64(q)).reshape(-1)
    assert q.size == m
    out = np.empty(n, dtype=np.float64)
    w = _work(n)
    base = (w.ctypes.data + 15) & ~15
    _c().oracle_csr_t_matvec(_p(x.rowptr), _p(x.colidx), _p(x.vals), _i(m), _i(n), _p(q),
                             _p(out), ctypes.c_void_p(base))
    return out


def csr_uv_dot(x: Csr, u, v):
    """P_k = U[i_k,:] . V[j_k,:] for every stored cell of X (nnz-vector)."""
    m, n = x.shape
    u, ldu = _rowmajor(u)
    v, ldv = _rowmajor(v)
    assert u.shape[0] == m and v.shape[0] == n and u.shape[1] == v.shape[1]
    p = np.empty(x.vals.size, dtype=np.float64)
    _c().oracle_csr_uv_dot(_p(x.rowptr), _p(x.colidx), _i(m), _p(u), _i(ldu), _p(v), _i(ldv),
                           _i(u.shape[1]), _p(p))
    return p


def matmul_nt(u, v):
    """U %*% t(V), dense (m x r) by (n x r) -> m x n."""
    u, ldu = _rowmajor(u)
    v, ldv = _rowmajor(v)
    assert u.shape[1] == v.shape[1]
    d = np.empty((u.shape[0], v.shape[0]), dtype=np.float64)
    _c().oracle_matmul_nt(_p(u), _i(u.shape[0]), _i(ldu), _p(v), _i(v.shape[0]), _i(ldv),
                          _i(u.shape[1]), _p(d))
    return d


def csr_row_sums(x: Csr, a):
    """rowSums of a matrix stored on X's pattern (a = its nnz-vector of values)."""
    a = np.ascontiguousarray(_f64(a)).reshape(-1)
    assert a.size == x.vals.size
    out = np.empty(x.shape[0], dtype=np.float64)
    _c().oracle_csr_row_sums(_p(x.rowptr), _i(x.shape[0]), _p(a), _p(out))
    return out


def csr_col_sums(x: Csr, a):
    """colSums of a matrix stored on X's pattern (a = its nnz-vector of values)."""
    a = np.ascontiguousarray(_f64(a)).reshape(-1)
    assert a.size == x.vals.size
    m, n = x.shape
    out = np.empty(n, dtype=np.float64)
    w = _work(n)
    base = (w.ctypes.data + 15) & ~15
    _c().oracle_csr_col_sums(_p(x.rowptr), _p(x.colidx), _i(m), _i(n), _p(a), _p(out),
                             ctypes.c_void_p(base))
    return out


def csr_matmul_dense(x: Csr, w, b):
    """W %*% B with W stored on X's pattern (w = its nnz-vector) and dense B (n x r) -> m x r."""
    m, n = x.shape
    w = np.ascontiguousarray(_f64(w)).reshape(-1)
    b, ldb = _rowmajor(b)
    assert w.size == x.vals.size and b.shape[0] == n
    o = np.empty((m, b.shape[1]), dtype=np.float64)
    _c().oracle_csr_matmul_dense(_p(x.rowptr), _p(x.colidx), _p(w), _i(m), _p(b), _i(ldb), _i(b.shape[1]), _p(o))
    return o


def csr_t_matmul_dense(x: Csr, w, b):
    """t(W) %*% B with W stored on X's pattern and dense B (m x r) -> n x r."""
    m, n = x.shape
    w = np.ascontiguousarray(_f64(w)).reshape(-1)
    b, ldb = _rowmajor(b)
    assert w.size == x.vals.size and b.shape[0] == m
    r = b.shape[1]
    o = np.empty((n, r), dtype=np.float64)
    wk = _work(n * r)
    base = (wk.ctypes.data + 15) & ~15
    _c().oracle_csr_t_matmul_dense(_p(x.rowptr), _p(x.colidx), _p(w), _i(m), _i(n), _p(b), _i(ldb), _i(r),
                                   _p(o), ctypes.c_void_p(base))
    return o


# ------------------------------------------------------------ CSR utilities ---

def csr_row_index(x: Csr):
    """Row index of every stored cell (nnz-vector, int64)."""
    return np.repeat(np.arange(x.shape[0], dtype=np.int64), np.diff(x.rowptr))


def csr_to_dense(x: Csr):
    """Dense m x n copy of X (tiny inputs only)."""
    d = np.zeros(x.shape, dtype=np.float64)
    d[csr_row_index(x), x.colidx] = x.vals
    return d
