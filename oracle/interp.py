"""Naive per-element interpreter of template expressions -- TEST INFRASTRUCTURE ONLY.

The second, independent evaluator: it follows the *fused* semantics of the
paper's skeletons (Sec. 2.2 "Runtime Integration": the skeleton walks the cells
/ rows / stored cells of the main input and calls the expression body once per
element) with pure-Python scalar loops and ``math.fsum`` for every aggregate.
Tiny inputs only.  The unfused plans are pinned against it: fused and unfused
evaluation must agree (Sec. 1).
"""
import math

import numpy as np


def _u(name, a):
    if name == "neg":
        return -a
    if name == "abs":
        return abs(a)
    if name == "sqrt":
        return math.sqrt(a) if a >= 0 else float("nan")
    if name == "exp":
        return math.exp(a)
    if name == "log":
        return math.log(a) if a > 0 else (float("-inf") if a == 0 else float("nan"))
    if name == "pow2":
        return a * a
    if name == "sign":
        return (a > 0) - (a < 0) + 0.0
    if name == "neq0":
        return 1.0 if a != 0 else 0.0
    if name == "sigmoid":
        return 1.0 / (1.0 + math.exp(-a))
    raise KeyError(name)


def _b(name, a, b):
    if name == "add":
        return a + b
    if name == "sub":
        return a - b
    if name == "mul":
        return a * b
    if name == "div":
        return a / b
    if name == "min":
        return min(a, b)
    if name == "max":
        return max(a, b)
    if name == "pow":
        return math.pow(a, b)
    if name == "lt":
        return float(a < b)
    if name == "le":
        return float(a <= b)
    if name == "gt":
        return float(a > b)
    if name == "ge":
        return float(a >= b)
    if name == "eq":
        return float(a == b)
    if name == "ne":
        return float(a != b)
    raise KeyError(name)


_UN = ("neg", "abs", "sqrt", "exp", "log", "pow2", "sign", "neq0", "sigmoid")
_BI = ("add", "sub", "mul", "div", "min", "max", "pow", "lt", "le", "gt", "ge", "eq", "ne")


def _side_at(sides, k, i, j):
    kind, arr = sides[k]
    a = np.asarray(arr, dtype=np.float64)
    if kind == "matrix":
        return float(a[i, j])
    if kind == "colvec":
        return float(a.reshape(-1)[i])
    if kind == "rowvec":
        return float(a.reshape(-1)[j])
    return float(a.reshape(-1)[0])


def _scalar_body(expr, a, sides, i, j, uvdot=None):
    st = []
    for tok in expr:
        name = tok[0]
        if name == "main":
            st.append(a)
        elif name == "side":
            st.append(_side_at(sides, tok[1], i, j))
        elif name == "const":
            st.append(float(tok[1]))
        elif name == "uvdot":
            st.append(uvdot)
        elif name in _UN:
            st.append(_u(name, st.pop()))
        elif name in _BI:
            y = st.pop()
            x = st.pop()
            st.append(_b(name, x, y))
        else:
            raise ValueError(tok)
    assert len(st) == 1
    return st[0]


def cell(expr, x, sides, agg):
    """Cell skeleton: body once per cell, then the aggregation variant."""
    x = np.asarray(x, dtype=np.float64)
    m, n = x.shape
    vals = [[_scalar_body(expr, float(x[i, j]), sides, i, j) for j in range(n)] for i in range(m)]
    if agg == "none":
        return np.array(vals, dtype=np.float64).reshape(m, n)
    if agg == "full":
        return np.array([math.fsum(v for r in vals for v in r)])
    if agg == "row":
        return np.array([math.fsum(r) for r in vals])
    if agg in ("col", "col_t"):
        return np.array([math.fsum(vals[i][j] for i in range(m)) for j in range(n)])
    raise ValueError(agg)


def magg(exprs, x, sides):
    """MAgg skeleton: one scan, k bodies per cell, k running sums."""
    x = np.asarray(x, dtype=np.float64)
    m, n = x.shape
    cols = [[] for _ in exprs]
    for i in range(m):
        for j in range(n):
            for k, e in enumerate(exprs):
                cols[k].append(_scalar_body(e, float(x[i, j]), sides, i, j))
    return np.array([math.fsum(c) for c in cols])


def _row_body(expr, xi, cols, n_cols, sides, i):
    """Row body for one row.  ``xi``: values of the row at column indices
    ``cols``.  Vector values are dicts {column: value} over ``cols`` (dense rows
    pass every column).  Returns ("V", dict) or ("S", float)."""
    st = []
    for tok in expr:
        name = tok[0]
        if name == "main":
            st.append(("V", dict(zip(cols, xi))))
        elif name == "side":
            kind = sides[tok[1]][0]
            if kind in ("matrix", "rowvec"):
                st.append(("V", {j: _side_at(sides, tok[1], i, j) for j in cols}))
            elif kind == "rhs":
                st.append(("M", np.asarray(sides[tok[1]][1], dtype=np.float64)))
            elif kind == "kvec":
                st.append(("K", [float(t) for t in np.asarray(sides[tok[1]][1], dtype=np.float64)[i]]))
            else:
                st.append(("S", _side_at(sides, tok[1], i, 0)))
        elif name == "const":
            st.append(("S", float(tok[1])))
        elif name in _UN:
            k, a = st.pop()
            if k == "V":
                st.append((k, {j: _u(name, v) for j, v in a.items()}))
            elif k == "K":
                st.append((k, [_u(name, v) for v in a]))
            else:
                st.append((k, _u(name, a)))
        elif name in _BI:
            kb, b = st.pop()
            ka, a = st.pop()
            if ka == "S" and kb == "S":
                st.append(("S", _b(name, a, b)))
            elif "K" in (ka, kb):
                assert "V" not in (ka, kb)
                kk = len(a) if ka == "K" else len(b)
                st.append(("K", [_b(name, a[t] if ka == "K" else a, b[t] if kb == "K" else b) for t in range(kk)]))
            else:
                st.append(("V", {j: _b(name, a[j] if ka == "V" else a, b[j] if kb == "V" else b)
                                 for j in cols}))
        elif name == "rowsum":
            k, a = st.pop()
            assert k in ("V", "K")
            st.append(("S", math.fsum(a.values() if k == "V" else a)))
        elif name == "dot":
            kb, b = st.pop()
            ka, a = st.pop()
            assert ka == kb and ka in ("V", "K")
            st.append(("S", math.fsum(a[j] * b[j] for j in (cols if ka == "V" else range(len(a))))))
        elif name == "matmult":       # vectMatMult: row vector times the n x k right-hand side
            kb, b = st.pop()
            ka, a = st.pop()
            assert ka == "V" and kb == "M"
            st.append(("K", [math.fsum(a[j] * float(b[j, t]) for j in cols) for t in range(b.shape[1])]))
        elif name == "outerk":        # vectOuterMultAdd: row (x) k-vector
            kb, b = st.pop()
            ka, a = st.pop()
            assert ka == "V" and kb == "K"
            st.append(("VK", (a, b)))
        else:
            raise ValueError(tok)
    assert len(st) == 1
    return st[0]


def row(expr, x, sides, agg):
    """Row skeleton over a dense matrix ``x`` (2-D array): body once per row."""
    x = np.asarray(x, dtype=np.float64)
    m, n = x.shape
    cols = list(range(n))
    res = [_row_body(expr, [float(t) for t in x[i]], cols, n, sides, i) for i in range(m)]
    return _row_aggregate(res, m, n, agg)


def row_sparse(expr, rowptr, colidx, vals, shape, sides, agg):
    """Row skeleton over CSR rows, evaluated densely: every row is expanded to
    all n columns (zeros included), so the result is the dense semantics that a
    sparse-safe program must reproduce."""
    m, n = shape
    dense = np.zeros((m, n))
    for i in range(m):
        for k in range(int(rowptr[i]), int(rowptr[i + 1])):
            dense[i, int(colidx[k])] = float(vals[k])
    return row(expr, dense, sides, agg)


def _row_aggregate(res, m, n, agg):
    if m == 0:
        return {"none": np.zeros((0, n)), "full": np.zeros(1), "row": np.zeros(0)}.get(agg, np.zeros(n))
    kind = res[0][0]
    if kind == "K":
        kk = len(res[0][1])
        if agg == "none":
            return np.array([r[1] for r in res]).reshape(m, kk)
        if agg in ("col", "col_t"):
            return np.array([math.fsum(r[1][t] for r in res) for t in range(kk)])
        if agg == "full":
            return np.array([math.fsum(v for r in res for v in r[1])])
        raise ValueError(agg)
    if kind == "VK":
        kk = len(res[0][1][1])
        if agg not in ("col", "col_t"):
            raise ValueError(agg)
        return np.array([[math.fsum(r[1][0][j] * r[1][1][t] for r in res) for t in range(kk)]
                         for j in range(n)]).reshape(n, kk)
    if kind == "S":
        if agg == "none":
            return np.array([r[1] for r in res])
        if agg == "full":
            return np.array([math.fsum(r[1] for r in res)])
        raise ValueError(agg)
    if agg == "none":
        return np.array([[r[1][j] for j in range(n)] for r in res]).reshape(m, n)
    if agg == "full":
        return np.array([math.fsum(v for r in res for v in r[1].values())])
    if agg == "row":
        return np.array([math.fsum(r[1].values()) for r in res])
    if agg in ("col", "col_t"):
        return np.array([math.fsum(r[1][j] for r in res) for j in range(n)])
    raise ValueError(agg)


def outer(expr, rowptr, colidx, vals, shape, u, v, sides, agg):
    """Outer skeleton: body once per stored cell (i, j) with a = X_ij and the
    inner product of U_i and V_j (Sec. 2.2, paragraph after the Outer listing)."""
    m, n = shape
    u = np.asarray(u, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    out, pos = [], []
    for i in range(m):
        for k in range(int(rowptr[i]), int(rowptr[i + 1])):
            j = int(colidx[k])
            d = math.fsum(float(u[i, t]) * float(v[j, t]) for t in range(u.shape[1]))
            out.append(_scalar_body(expr, float(vals[k]), sides, i, j, uvdot=d))
            pos.append((i, j))
    r = u.shape[1]
    if agg == "right_mm":      # I_i += w_ij * V_j
        return np.array([[math.fsum(w * float(v[j, t]) for w, (ii, j) in zip(out, pos) if ii == i)
                          for t in range(r)] for i in range(m)]).reshape(m, r)
    if agg == "left_mm":       # I_j += w_ij * U_i
        return np.array([[math.fsum(w * float(u[i, t]) for w, (i, jj) in zip(out, pos) if jj == j)
                          for t in range(r)] for j in range(n)]).reshape(n, r)
    if agg == "none":
        return np.array(out, dtype=np.float64)
    if agg == "full":
        return np.array([math.fsum(out)])
    raise ValueError(agg)
