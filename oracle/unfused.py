"""Operator-at-a-time evaluation of template expressions -- TEST INFRASTRUCTURE ONLY.

A fused operator computes exactly what the chain of basic operators it replaces
computes (Sec. 1, "Fusion Opportunities": fusion removes intermediates and
scans, not arithmetic).  So the reference result of an expression is the plain
definition: walk the postfix expression, execute ONE basic operator of
``oracle.ops`` per token over whole matrices, and materialise every
intermediate -- the paper's "Base" plan (Sec. 5.1).

Expressions are symbolic postfix lists of tuples:
    ("main",)            the template's main input X (cell / row / stored cell)
    ("side", k)          side input k (Table 1: the list Y of side inputs)
    ("const", c)         literal scalar
    ("uvdot",)           Outer only: U[i,:] . V[j,:] at the stored cell (i, j)
    (name,)              element-wise unary / binary operator, see ``oracle.ops``
    ("rowsum",)          Row only: sum over the columns of a row vector (or over the
                         entries of a k-vector)
    ("dot",)             Row only: inner product of two row vectors (or two k-vectors)
    ("matmult",)         Row only: row vector times a "rhs" side (n x k) -> k-vector
    ("outerk",)          Row only, last token: row vector (x) k-vector, an n x k
                         matrix per row that is summed over the rows (col / col_t)
Side inputs are ``(kind, array)`` pairs with kind in
    "matrix" (m x n), "colvec" (m, indexed by row), "rowvec" (n, indexed by
    column), "scalar", and for Row bodies "rhs" (n x k, the right-hand side of
    "matmult") and "kvec" (m x k: one k-vector per row).
Aggregation variants (Table 1): "none", "full", "row", "col", "col_t".
"""
import numpy as np

from . import ops

_ZERO_PRESERVING_UNARY = {"neg", "abs", "sqrt", "pow2", "sign", "neq0"}


def _side_dense(kind, arr, m, n):
    """Side input as an array that broadcasts against an m x n matrix."""
    a = np.asarray(arr, dtype=np.float64)
    if kind == "matrix":
        assert a.shape == (m, n), (a.shape, (m, n))
        return a
    if kind == "colvec":
        assert a.size == m
        return a.reshape(m, 1)
    if kind == "rowvec":
        assert a.size == n
        return a.reshape(1, n)
    if kind == "scalar":
        assert a.size == 1
        return a.reshape(())
    raise ValueError("unknown side kind %r" % (kind,))


def _aggregate_dense(r, m, n, agg):
    """Apply a Table-1 aggregation variant to a (broadcastable) m x n result."""
    full = np.array(np.broadcast_to(r, (m, n)), dtype=np.float64)   # materialise
    if agg == "none":
        return full
    if agg == "full":
        return np.array([ops.sum_full(full)])
    if agg == "row":
        return ops.row_sums(full) if n > 0 else np.zeros(m)
    if agg in ("col", "col_t"):
        return ops.col_sums(full) if m > 0 else np.zeros(n)
    raise ValueError("unknown aggregation %r" % (agg,))


# ---------------------------------------------------------------- Cell, MAgg ---

def _eval_cells(expr, x, sides):
    m, n = x.shape
    st = []
    for tok in expr:
        name = tok[0]
        if name == "main":
            st.append(x)
        elif name == "side":
            kind, arr = sides[tok[1]]
            st.append(_side_dense(kind, arr, m, n))
        elif name == "const":
            st.append(np.float64(tok[1]))
        elif name in ops.UNARY_NAMES:
            a = st.pop()
            st.append(ops.ew_unary(name, a))
        elif name in ops.BINARY_NAMES:
            b = st.pop()
            a = st.pop()
            st.append(ops.ew_binary(name, a, b))
        else:
            raise ValueError("token %r is not valid in a Cell expression" % (tok,))
    if len(st) != 1:
        raise ValueError("expression leaves %d values on the stack" % len(st))
    return st[0]


def cell(expr, x, sides, agg):
    """Cell template (Table 1; Sec. 2.2 Cell listing): per-cell chain over dense X,
    then the aggregation variant.  Returns a float64 array (shape by variant)."""
    x = np.asarray(x, dtype=np.float64)
    m, n = x.shape
    return _aggregate_dense(_eval_cells(expr, x, sides), m, n, agg)


def magg(exprs, x, sides):
    """MAgg template (Table 1; Fig. 1c; Sec. 5.2 "Multi-Aggregate Operations"):
    k full aggregates, each computed on its own, unfused; returns k values."""
    return np.array([cell(e, x, sides, "full")[0] for e in exprs])


# ----------------------------------------------------------------------- Row ---

def row_dense(expr, x, sides, agg):
    """Row template over a dense main input (Table 1; Sec. 2.2 Row listing).

    Values are row vectors ("V": broadcastable to m x n), per-row scalars ("S":
    shape (m,1) or ()), per-row k-vectors ("K": m x k; products with an n x k
    right-hand side, vectMatMult) or the right-hand side itself ("M").  Returns an
    array shaped by the variant and the kind of the result:
      V: none -> m x n; row -> m; col / col_t -> n; full -> 1
      S: none -> m; full -> 1
      K: none -> m x k; col / col_t -> k (sums over the rows); full -> 1
      row (x) k-vector ("outerk"): col / col_t -> n x k = t(V-part) %*% K-part
         (vectOuterMultAdd; the COL_AGG_B1_T variant of the Row listing)
    """
    x = np.asarray(x, dtype=np.float64)
    m, n = x.shape
    st = []   # (kind, array)
    outer = None
    for pos, tok in enumerate(expr):
        name = tok[0]
        if outer is not None:
            raise ValueError("outerk must be the last token")
        if name == "main":
            st.append(("V", x))
        elif name == "side":
            kind, arr = sides[tok[1]]
            if kind == "rhs":
                a = np.asarray(arr, dtype=np.float64)
                assert a.ndim == 2 and a.shape[0] == n
                st.append(("M", a))
            elif kind == "kvec":
                a = np.asarray(arr, dtype=np.float64)
                assert a.ndim == 2 and a.shape[0] == m
                st.append(("K", a))
            else:
                a = _side_dense(kind, arr, m, n)
                st.append(("V" if kind in ("matrix", "rowvec") else "S", a))
        elif name == "const":
            st.append(("S", np.float64(tok[1])))
        elif name in ops.UNARY_NAMES:
            k, a = st.pop()
            if k == "M":
                raise ValueError("a right-hand side can only be consumed by matmult")
            st.append((k, ops.ew_unary(name, a)))
        elif name in ops.BINARY_NAMES:
            kb, b = st.pop()
            ka, a = st.pop()
            kinds = {ka, kb}
            if "M" in kinds or kinds == {"V", "K"}:
                raise ValueError("operands of %r do not conform" % name)
            st.append(("V" if "V" in kinds else "K" if "K" in kinds else "S", ops.ew_binary(name, a, b)))
        elif name == "rowsum":
            k, a = st.pop()
            if k == "K":
                st.append(("S", ops.row_sums(np.array(a)).reshape(m, 1)))
            elif k == "V":
                full = np.array(np.broadcast_to(a, (m, n)))
                st.append(("S", ops.row_sums(full).reshape(m, 1)))
            else:
                raise ValueError("rowsum of a scalar")
        elif name == "dot":
            kb, b = st.pop()
            ka, a = st.pop()
            if ka == "K" and kb == "K":
                st.append(("S", ops.row_sums(ops.ew_binary("mul", a, b)).reshape(m, 1)))
            elif ka == "V" and kb == "V":
                t = np.array(np.broadcast_to(ops.ew_binary("mul", a, b), (m, n)))
                st.append(("S", ops.row_sums(t).reshape(m, 1)))
            else:
                raise ValueError("dot needs two row vectors or two k-vectors")
        elif name == "matmult":
            kb, b = st.pop()
            ka, a = st.pop()
            if ka != "V" or kb != "M":
                raise ValueError("matmult needs a row vector and a right-hand side")
            st.append(("K", ops.matmul(np.array(np.broadcast_to(a, (m, n))), b)))
        elif name == "outerk":
            kb, b = st.pop()
            ka, a = st.pop()
            if ka != "V" or kb != "K":
                raise ValueError("outerk needs a row vector and a k-vector")
            outer = (np.array(np.broadcast_to(a, (m, n))), np.array(b))
        else:
            raise ValueError("token %r is not valid in a Row expression" % (tok,))
    if outer is not None:
        if st:
            raise ValueError("expression leaves values on the stack")
        if agg not in ("col", "col_t"):
            raise ValueError("a row (x) k-vector result needs the column aggregate")
        return ops.t_matmul(outer[0], outer[1])
    if len(st) != 1:
        raise ValueError("expression leaves %d values on the stack" % len(st))
    kind, r = st[0]
    if kind == "M":
        raise ValueError("a right-hand side is not a result")
    if kind == "V":
        return _aggregate_dense(r, m, n, agg)
    if kind == "K":
        r = np.array(r, dtype=np.float64)
        if agg == "none":
            return r
        if agg in ("col", "col_t"):
            return ops.col_sums(r)
        if agg == "full":
            return np.array([ops.sum_full(r)])
        raise ValueError("aggregation %r is not defined for a k-vector result" % (agg,))
    per_row = np.array(np.broadcast_to(np.asarray(r).reshape(-1, 1) if np.ndim(r) else r, (m, 1)),
                       dtype=np.float64).reshape(m)
    if agg == "none":
        return per_row
    if agg == "full":
        return np.array([ops.sum_full(per_row)])
    raise ValueError("aggregation %r needs a row-vector result" % (agg,))


def row_csr(expr, x: ops.Csr, sides, agg):
    """Row template over a CSR main input: the sparse-safe binding (Sec. 2.2
    "Template Types": a sparse-safe template binds only to the non-zeros).

    Row-vector values are carried on X's pattern (one value per stored cell); a
    value is usable that way only if it is zero wherever X has no stored cell,
    which is tracked per value.  Dense-valued vectors (side inputs) are gathered
    at the stored positions and may only be consumed by an operator that makes
    the result zero-preserving again (e.g. multiply with X).  Programs that are
    not sparse-safe raise ValueError.
    Products with an n x k right-hand side (vectMatMult over the stored cells of a
    row) give per-row k-vectors ("K", m x k); "outerk" (vectOuterMultAdd with the
    column aggregate) sums row (x) k-vector products into n x k.  Both need a
    zero-preserving row-vector operand.
    Returns: none -> nnz-vector on X's pattern (V), m (S) or m x k (K); row -> m;
    col / col_t -> n (V), k (K) or n x k (outerk); full -> 1.
    """
    m, n = x.shape
    rows = ops.csr_row_index(x)
    st = []   # ("V", nnz-array, zero_preserving) | ("S", array (m,) or 0-d) | ("K", m x k) | ("M", n x k)
    outer = None

    def col1(k, a):        # per-row scalar next to a k-vector: (m,) -> (m, 1)
        a = np.asarray(a, dtype=np.float64)
        return a.reshape(m, 1) if (k == "S" and a.ndim == 1) else a

    def expand(k, a):      # per-row scalar -> per stored cell
        a = np.asarray(a, dtype=np.float64)
        return a if (k == "V" or a.ndim == 0) else a[rows]

    for tok in expr:
        name = tok[0]
        if outer is not None:
            raise ValueError("outerk must be the last token")
        if name == "main":
            st.append(("V", x.vals, True))
        elif name == "side":
            kind, arr = sides[tok[1]]
            a = np.asarray(arr, dtype=np.float64)
            if kind == "matrix":
                assert a.shape == (m, n)
                st.append(("V", a[rows, x.colidx], False))
            elif kind == "rowvec":
                assert a.size == n
                st.append(("V", a.reshape(-1)[x.colidx], False))
            elif kind == "colvec":
                assert a.size == m
                st.append(("S", a.reshape(m), None))
            elif kind == "scalar":
                st.append(("S", a.reshape(()), None))
            elif kind == "rhs":
                assert a.ndim == 2 and a.shape[0] == n
                st.append(("M", a, None))
            elif kind == "kvec":
                assert a.ndim == 2 and a.shape[0] == m
                st.append(("K", a, None))
            else:
                raise ValueError(kind)
        elif name == "const":
            st.append(("S", np.float64(tok[1]), None))
        elif name in ops.UNARY_NAMES:
            k, a, z = st.pop()
            if k == "M":
                raise ValueError("a right-hand side can only be consumed by matmult")
            zz = (z and name in _ZERO_PRESERVING_UNARY) if k == "V" else None
            st.append((k, ops.ew_unary(name, a), zz))
        elif name in ops.BINARY_NAMES:
            kb, b, zb = st.pop()
            ka, a, za = st.pop()
            if ka == "S" and kb == "S":
                st.append(("S", ops.ew_binary(name, a, b), None))
                continue
            if "M" in (ka, kb) or {ka, kb} == {"V", "K"}:
                raise ValueError("operands of %r do not conform" % name)
            if "K" in (ka, kb):
                st.append(("K", ops.ew_binary(name, col1(ka, a), col1(kb, b)), None))
                continue
            if name == "mul":
                z = bool(za) or bool(zb)
            elif name in ("add", "sub"):
                z = ka == "V" and kb == "V" and za and zb
            elif name == "div":
                z = ka == "V" and bool(za)
            else:
                z = False
            st.append(("V", ops.ew_binary(name, expand(ka, a), expand(kb, b)), z))
        elif name in ("rowsum", "dot"):
            if name == "dot":
                kb, b, zb = st.pop()
                ka, a, za = st.pop()
                if ka == "K" and kb == "K":
                    st.append(("S", ops.row_sums(ops.ew_binary("mul", a, b)), None))
                    continue
                if ka != "V" or kb != "V":
                    raise ValueError("dot needs two row vectors or two k-vectors")
                a, z, k = ops.ew_binary("mul", a, b), bool(za) or bool(zb), "V"
            else:
                k, a, z = st.pop()
                if k == "K":
                    st.append(("S", ops.row_sums(np.array(a, dtype=np.float64)), None))
                    continue
            if k != "V":
                raise ValueError("rowsum of a scalar")
            if not z:
                raise ValueError("not sparse-safe: row aggregate of a dense-valued vector")
            st.append(("S", ops.csr_row_sums(x, a), None))
        elif name == "matmult":
            kb, b, _ = st.pop()
            ka, a, za = st.pop()
            if ka != "V" or kb != "M":
                raise ValueError("matmult needs a row vector and a right-hand side")
            if not za:
                raise ValueError("not sparse-safe: product of a dense-valued vector with a right-hand side")
            st.append(("K", ops.csr_matmul_dense(x, np.array(np.broadcast_to(a, x.vals.shape)), b), None))
        elif name == "outerk":
            kb, b, _ = st.pop()
            ka, a, za = st.pop()
            if ka != "V" or kb != "K":
                raise ValueError("outerk needs a row vector and a k-vector")
            if not za:
                raise ValueError("not sparse-safe: outer product of a dense-valued vector")
            outer = (np.array(np.broadcast_to(a, x.vals.shape)), np.array(b, dtype=np.float64))
        else:
            raise ValueError("token %r is not valid in a Row expression" % (tok,))
    if outer is not None:
        if st:
            raise ValueError("expression leaves values on the stack")
        if agg not in ("col", "col_t"):
            raise ValueError("a row (x) k-vector result needs the column aggregate")
        return ops.csr_t_matmul_dense(x, outer[0], outer[1])
    if len(st) != 1:
        raise ValueError("expression leaves %d values on the stack" % len(st))
    kind, r, z = st[0]
    if kind == "M":
        raise ValueError("a right-hand side is not a result")
    if kind == "K":
        r = np.array(r, dtype=np.float64)
        if agg == "none":
            return r
        if agg in ("col", "col_t"):
            return ops.col_sums(r)
        if agg == "full":
            return np.array([ops.sum_full(r)])
        raise ValueError("aggregation %r is not defined for a k-vector result" % (agg,))
    if kind == "S":
        per_row = np.array(np.broadcast_to(r, (m,)), dtype=np.float64)
        if agg == "none":
            return per_row
        if agg == "full":
            return np.array([ops.sum_full(per_row)])
        raise ValueError("aggregation %r needs a row-vector result" % (agg,))
    if not z:
        raise ValueError("not sparse-safe: result is not zero where X is zero")
    r = np.array(np.broadcast_to(r, x.vals.shape), dtype=np.float64)
    if agg == "none":
        return r
    if agg == "full":
        return np.array([ops.sum_full(r)])
    if agg == "row":
        return ops.csr_row_sums(x, r)
    if agg in ("col", "col_t"):
        return ops.csr_col_sums(x, r)
    raise ValueError("unknown aggregation %r" % (agg,))


def cell_csr(expr, x: ops.Csr, sides, agg):
    """Cell template over a sparse main input (Fig. 8b; Sec. 5.2 "Cell Operations": X is
    the sparse driver): the sparse-safe body is evaluated over nnz-vectors on X's
    pattern -- a Row body without row aggregates.  Shapes as for ``row_csr``."""
    for tok in expr:
        if tok[0] in ("rowsum", "dot", "uvdot"):
            raise ValueError("token %r is not valid in a Cell expression" % (tok,))
    return row_csr(expr, x, sides, agg)


def magg_csr(exprs, x: ops.Csr, sides):
    """MAgg over a sparse main input (Fig. 8d): k full aggregates, each on its own."""
    return np.array([cell_csr(e, x, sides, "full")[0] for e in exprs])


# --------------------------------------------------------------------- Outer ---

def outer(expr, x: ops.Csr, u, v, sides, agg):
    """Outer template (Table 1; Sec. 2.2 Outer listing and the paragraph after
    it): binds to every stored cell X_ij, the rows U_i and V_j and dense side
    inputs; the chain is evaluated over nnz-vectors, never over m x n.

    agg "full" -> 1 value; "none" -> nnz-vector on X's pattern;
    "right_mm" -> m x r: the body values W (on X's pattern) times V, i.e. row i
    accumulates w_ij * V_j (Sec. 2.2, paragraph after the Outer listing);
    "left_mm" -> n x r: t(W) times U, i.e. row j accumulates w_ij * U_i (the
    mirrored variant of Table 1).
    """
    m, n = x.shape
    rows = ops.csr_row_index(x)
    st = []
    for tok in expr:
        name = tok[0]
        if name == "main":
            st.append(x.vals)
        elif name == "uvdot":
            st.append(ops.csr_uv_dot(x, u, v))
        elif name == "side":
            kind, arr = sides[tok[1]]
            a = np.asarray(arr, dtype=np.float64)
            if kind == "matrix":
                assert a.shape == (m, n)
                st.append(a[rows, x.colidx])
            elif kind == "colvec":
                st.append(a.reshape(m)[rows])
            elif kind == "rowvec":
                st.append(a.reshape(n)[x.colidx])
            elif kind == "scalar":
                st.append(a.reshape(()))
            else:
                raise ValueError(kind)
        elif name == "const":
            st.append(np.float64(tok[1]))
        elif name in ops.UNARY_NAMES:
            st.append(ops.ew_unary(name, st.pop()))
        elif name in ops.BINARY_NAMES:
            b = st.pop()
            a = st.pop()
            st.append(ops.ew_binary(name, a, b))
        else:
            raise ValueError("token %r is not valid in an Outer expression" % (tok,))
    if len(st) != 1:
        raise ValueError("expression leaves %d values on the stack" % len(st))
    r = np.array(np.broadcast_to(st[0], x.vals.shape), dtype=np.float64)
    if agg == "none":
        return r
    if agg == "full":
        return np.array([ops.sum_full(r)])
    if agg == "right_mm":
        return ops.csr_matmul_dense(x, r, v)
    if agg == "left_mm":
        return ops.csr_t_matmul_dense(x, r, u)
    raise ValueError("unknown aggregation %r" % (agg,))
