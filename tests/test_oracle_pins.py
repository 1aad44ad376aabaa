"""Pins for the oracle's template evaluators and the five workload plans (no GPU).

The paper prints no numeric result of any fused expression, so each plan is
pinned by closed forms, integer-exact cases, brute force on tiny inputs
(``oracle.interp``: fused semantics, pure-Python loops + fsum), library
routines (numpy / scipy) and the invariants the paper states (fused == unfused,
Sec. 1; a multi-aggregate equals its aggregates computed one by one, Sec. 5.2).
"""
import math

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ops, plans, unfused, interp
import workloads as W
from exprgen import random_scalar_expr, random_row_expr

CELL_XYZ = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
ROW_TXWXV = [("main",), ("side", 0), ("dot",), ("side", 1), ("mul",), ("main",), ("mul",)]
ROW_TXXV = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
OUTER_LOG = [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]


def _rng(s):
    return np.random.default_rng(s)


def _csr(m, n, d, seed):
    rp, ci, v = W.csr_bernoulli(m, n, d, seed)
    return ops.make_csr(rp, ci, v, (m, n))


# ----------------------------------------------------------------------- Cell ---

@pytest.mark.parametrize("c", [0.5, 2.0])
def test_cell_constant_closed_form(c):
    m, n = 123, 77
    x = np.full((m, n), c)
    assert plans.cell_sum_xyz(x, x, x)[0] == m * n * c ** 3
    assert unfused.cell(CELL_XYZ, x, [("matrix", x), ("matrix", x)], "full")[0] == m * n * c ** 3


def test_cell_integer_exact():
    m, n = 211, 97
    x = np.ones((m, n))
    y = np.repeat(np.arange(m, dtype=np.float64)[:, None], n, 1)
    z = np.repeat(np.arange(n, dtype=np.float64)[None, :], m, 0)
    assert plans.cell_sum_xyz(x, y, z)[0] == (m * (m - 1) // 2) * (n * (n - 1) // 2)


def test_cell_brute_force_and_numpy():
    r = _rng(1)
    x, y, z = r.uniform(size=(3, 7, 8))
    ref = math.fsum(x[i, j] * y[i, j] * z[i, j] for i in range(7) for j in range(8))
    assert abs(plans.cell_sum_xyz(x, y, z)[0] - ref) <= 4 * np.spacing(ref)
    X, Y, Z = r.uniform(size=(3, 300, 1000))
    np.testing.assert_allclose(plans.cell_sum_xyz(X, Y, Z)[0], (X * Y * Z).sum(), rtol=1e-13)
    np.testing.assert_allclose(unfused.cell(CELL_XYZ, X, [("matrix", Y), ("matrix", Z)], "full"),
                               plans.cell_sum_xyz(X, Y, Z), rtol=0, atol=0)


def test_cell_variants_and_side_kinds():
    r = _rng(2)
    m, n = 9, 6
    x, y = r.normal(size=(2, m, n))
    cv, rv = r.normal(size=m), r.normal(size=n)
    # the ALS-CG update of Sec. 2.2 (Cell listing): Y + X * 1e-6 * colvec, no aggregation
    expr = [("side", 0), ("main",), ("const", 1e-6), ("mul",), ("side", 1), ("mul",), ("add",)]
    sides = [("matrix", y), ("colvec", cv)]
    got = unfused.cell(expr, x, sides, "none")
    np.testing.assert_allclose(got, y + x * 1e-6 * cv[:, None], rtol=1e-15)
    e2 = [("main",), ("side", 0), ("mul",), ("side", 1), ("add",)]
    s2 = [("rowvec", rv), ("scalar", np.array(0.75))]
    full = x * rv[None, :] + 0.75
    np.testing.assert_allclose(unfused.cell(e2, x, s2, "none"), full, rtol=1e-15)
    np.testing.assert_allclose(unfused.cell(e2, x, s2, "row"), full.sum(1), rtol=1e-13)
    np.testing.assert_allclose(unfused.cell(e2, x, s2, "col"), full.sum(0), rtol=1e-13)
    np.testing.assert_allclose(unfused.cell(e2, x, s2, "full"), [full.sum()], rtol=1e-13)
    for agg in ("none", "row", "col", "full"):
        np.testing.assert_allclose(unfused.cell(e2, x, s2, agg), interp.cell(e2, x, s2, agg), rtol=1e-14, atol=1e-15)


# ----------------------------------------------------------------------- MAgg ---

def test_magg_constants_and_checkerboard():
    m, n = 50, 31
    a, b, c = 0.5, 4.0, -2.0
    x, y, z = np.full((m, n), a), np.full((m, n), b), np.full((m, n), c)
    assert plans.magg_xy_xz_xx(x, y, z).tolist() == [m * n * a * b, m * n * a * c, m * n * a * a]
    i, j = np.indices((m, n))
    chk = np.where((i + j) % 2 == 0, 1.0, -1.0)
    got = plans.magg_xy_xz_xx(chk, np.ones((m, n)), chk)
    assert got.tolist() == [0.0, float(m * n), float(m * n)]     # m*n even here
    g2 = plans.magg_xy_xz_xx(chk[:, :30][:49], np.ones((49, 30)), chk[:49, :30])
    assert g2.tolist() == [0.0, 49 * 30.0, 49 * 30.0]
    g3 = plans.magg_xy_xz_xx(chk[:49], np.ones((49, n)), chk[:49])
    assert g3.tolist() == [1.0, 49.0 * n, 49.0 * n]              # odd cell count: one +1 left over


def test_magg_equals_separate_aggregates():
    r = _rng(3)
    x, y, z = r.uniform(-1, 1, size=(3, 200, 300))
    exprs = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)], [("main",), ("pow2",)]]
    sides = [("matrix", y), ("matrix", z)]
    got = plans.magg_xy_xz_xx(x, y, z)
    np.testing.assert_array_equal(got, unfused.magg(exprs, x, sides))
    np.testing.assert_allclose(got, [(x * y).sum(), (x * z).sum(), (x * x).sum()], rtol=1e-11)
    xs, ys, zs = x[:6, :5], y[:6, :5], z[:6, :5]
    np.testing.assert_allclose(plans.magg_xy_xz_xx(xs, ys, zs),
                               interp.magg(exprs, xs, [("matrix", ys), ("matrix", zs)]), rtol=1e-14)


# ------------------------------------------------------------------ Row dense ---

def test_row_dense_ones_and_one_hot():
    m, n = 64, 10
    out = plans.row_tx_w_xv(np.ones((m, n)), np.ones(n), np.ones(m))
    assert out.tolist() == [float(m * n)] * n
    r = _rng(4)
    c = r.integers(0, n, size=m)
    x = np.zeros((m, n))
    x[np.arange(m), c] = 1.0
    v, w = r.normal(size=n), r.uniform(size=m)
    ref = [v[j] * math.fsum(w[c == j]) for j in range(n)]
    np.testing.assert_allclose(plans.row_tx_w_xv(x, v, w), ref, rtol=1e-14, atol=1e-15)


def test_row_dense_invariants_and_numpy():
    r = _rng(5)
    m, n = 500, 37
    x, v, u, w = r.normal(size=(m, n)), r.normal(size=n), r.normal(size=n), r.uniform(size=m)
    fv, fu = plans.row_tx_w_xv(x, v, w), plans.row_tx_w_xv(x, u, w)
    np.testing.assert_allclose(fv, x.T @ (w * (x @ v)), rtol=1e-11, atol=1e-11)
    quad = math.fsum(w[i] * float(x[i] @ v) ** 2 for i in range(m))
    assert v @ fv >= 0 and abs(v @ fv - quad) <= 1e-11 * quad
    assert abs(u @ fv - v @ fu) <= 1e-11 * abs(u @ fv)
    sides = [("rowvec", v), ("colvec", w)]
    np.testing.assert_allclose(unfused.row_dense(ROW_TXWXV, x, sides, "col_t"), fv, rtol=1e-13, atol=1e-13)
    xs, ws = x[:7, :5], w[:7]
    ss = [("rowvec", v[:5]), ("colvec", ws)]
    np.testing.assert_allclose(plans.row_tx_w_xv(xs, v[:5], ws), interp.row(ROW_TXWXV, xs, ss, "col_t"), rtol=1e-13, atol=1e-14)


# -------------------------------------------------------------------- Row CSR ---

def test_row_csr_vs_dense_scipy_and_permutation():
    m, n = 400, 60
    x = _csr(m, n, 0.07, 21)
    v = _rng(6).normal(size=n)
    got = plans.row_csr_tx_xv(x, v)
    d = ops.csr_to_dense(x)
    np.testing.assert_allclose(got, plans.row_tx_w_xv(d, v, np.ones(m)), rtol=1e-14, atol=1e-15)
    s = sp.csr_matrix((x.vals, x.colidx, x.rowptr), shape=(m, n))
    np.testing.assert_allclose(got, s.T @ (s @ v), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(unfused.row_csr(ROW_TXXV, x, [("rowvec", v)], "col_t"), got, rtol=1e-13, atol=1e-14)
    # column permutation: permuting X's columns and v alike permutes the output
    perm = _rng(7).permutation(n)
    inv = np.argsort(perm)
    sp2 = sp.csr_matrix(s[:, perm])
    sp2.sort_indices()
    x2 = ops.make_csr(sp2.indptr, sp2.indices, sp2.data, (m, n))
    np.testing.assert_allclose(plans.row_csr_tx_xv(x2, v[perm])[inv], got, rtol=1e-13, atol=1e-14)


def test_row_csr_empty_rows_and_empty_matrix():
    m, n = 20, 9
    x = ops.make_csr(np.zeros(m + 1, dtype=np.int64), np.zeros(0, np.int32), np.zeros(0), (m, n))
    assert plans.row_csr_tx_xv(x, np.ones(n)).tolist() == [0.0] * n
    # rows 0, 3 and the last are empty
    rp = np.array([0, 0, 2, 3, 3, 5, 5], dtype=np.int64)
    ci = np.array([1, 4, 0, 2, 3], dtype=np.int32)
    va = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    x = ops.make_csr(rp, ci, va, (6, 5))
    v = np.array([1.0, 10.0, 100.0, 1000.0, 10000.0])
    q = [0.0, 20010.0, 3.0, 0.0, 5400.0, 0.0]
    ref = [3 * q[2], 1 * q[1], 4 * q[4], 5 * q[4], 2 * q[1]]
    assert plans.row_csr_tx_xv(x, v).tolist() == ref


# ---------------------------------------------------------------------- Outer ---

def test_outer_closed_forms():
    m, n, r = 50, 40, 100
    rp, ci, _ = W.csr_bernoulli(m, n, 0.1, 31)
    x = ops.make_csr(rp, ci, np.ones(ci.size), (m, n))
    u, v = np.ones((m, r)), np.ones((n, r))
    np.testing.assert_allclose(plans.outer_sum_x_log_uv(x, u, v)[0], ci.size * math.log(100.0), rtol=1e-15)
    a, b = 0.5, 3.0
    vals = _rng(8).uniform(size=ci.size)
    x = ops.make_csr(rp, ci, vals, (m, n))
    ref = math.log(r * a * b + 1e-15) * math.fsum(vals)
    np.testing.assert_allclose(plans.outer_sum_x_log_uv(x, np.full((m, r), a), np.full((n, r), b))[0], ref, rtol=1e-14)
    # rows of U that are zero: each of their stored cells contributes x * log(1e-15)
    u = np.ones((m, r))
    u[::2] = 0.0
    rows = ops.csr_row_index(x)
    ref = math.fsum(vals[k] * (math.log(1e-15) if rows[k] % 2 == 0 else math.log(100.0 + 1e-15)) for k in range(ci.size))
    np.testing.assert_allclose(plans.outer_sum_x_log_uv(x, u, np.ones((n, r)))[0], ref, rtol=1e-14)


def test_outer_vs_dense_plan_and_interp():
    m, n, r = 23, 19, 7
    g = _rng(9)
    u, v = g.uniform(size=(m, r)), g.uniform(size=(n, r))
    for dens in (0.15, 1.0):
        x = _csr(m, n, dens, 32)
        got = plans.outer_sum_x_log_uv(x, u, v)
        np.testing.assert_allclose(got, plans.outer_sum_x_log_uv_dense(ops.csr_to_dense(x), u, v), rtol=1e-13)
        np.testing.assert_allclose(got, interp.outer(OUTER_LOG, x.rowptr, x.colidx, x.vals, x.shape, u, v, [], "full"), rtol=1e-13)
        np.testing.assert_array_equal(got, unfused.outer(OUTER_LOG, x, u, v, [], "full"))
        rows = ops.csr_row_index(x)
        ref = (x.vals * np.log((u[rows] * v[x.colidx]).sum(1) + 1e-15)).sum()
        np.testing.assert_allclose(got[0], ref, rtol=1e-13)
    assert plans.outer_sum_x_log_uv(_csr(m, n, 1.0, 1), u, v).shape == (1,)
    empty = ops.make_csr(np.zeros(m + 1, np.int64), np.zeros(0, np.int32), np.zeros(0), (m, n))
    assert plans.outer_sum_x_log_uv(empty, u, v)[0] == 0.0


# ------------------------------------------------ descriptor machinery (random) ---

def _sides(rng, kinds, m, n):
    out = []
    for k in kinds:
        if k == "matrix":
            out.append((k, rng.uniform(-1.5, 1.5, size=(m, n))))
        elif k == "colvec":
            out.append((k, rng.uniform(-1.5, 1.5, size=m)))
        elif k == "rowvec":
            out.append((k, rng.uniform(-1.5, 1.5, size=n)))
        else:
            out.append((k, np.array(rng.uniform(-1.5, 1.5))))
    return out


@pytest.mark.parametrize("seed", range(25))
def test_random_cell_expressions_unfused_equals_interp(seed):
    rng = _rng(1000 + seed)
    m, n = int(rng.integers(1, 7)), int(rng.integers(1, 7))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    x[rng.random((m, n)) < 0.2] = 0.0
    expr = random_scalar_expr(rng, len(kinds))
    for agg in ("none", "row", "col", "full"):
        np.testing.assert_allclose(unfused.cell(expr, x, sides, agg), interp.cell(expr, x, sides, agg),
                                   rtol=1e-12, atol=1e-13, equal_nan=True)


@pytest.mark.parametrize("seed", range(25))
def test_random_row_expressions_unfused_equals_interp(seed):
    rng = _rng(2000 + seed)
    m, n = int(rng.integers(1, 7)), int(rng.integers(1, 8))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    want = "V" if seed % 3 else "S"
    expr = random_row_expr(rng, kinds, depth=3, want=want)
    for agg in (("none", "row", "col", "col_t", "full") if want == "V" else ("none", "full")):
        np.testing.assert_allclose(unfused.row_dense(expr, x, sides, agg), interp.row(expr, x, sides, agg),
                                   rtol=1e-11, atol=1e-12, equal_nan=True)


@pytest.mark.parametrize("seed", range(25))
def test_random_sparse_safe_row_expressions(seed):
    """CSR evaluation over stored cells == dense semantics over all cells."""
    rng = _rng(3000 + seed)
    m, n = int(rng.integers(1, 8)), int(rng.integers(1, 9))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = _csr(m, n, 0.4, 3000 + seed)
    want = "V" if seed % 3 else "S"
    expr = random_row_expr(rng, kinds, depth=3, want=want, sparse_safe=True)
    for agg in (("none", "row", "col", "col_t", "full") if want == "V" else ("none", "full")):
        got = unfused.row_csr(expr, x, sides, agg)
        ref = interp.row_sparse(expr, x.rowptr, x.colidx, x.vals, x.shape, sides, agg)
        if want == "V" and agg == "none":      # compare on the pattern, and zero elsewhere
            dense = np.zeros((m, n))
            dense[ops.csr_row_index(x), x.colidx] = got
            got = dense
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12, equal_nan=True)


def test_row_csr_rejects_programs_that_are_not_sparse_safe():
    x = _csr(6, 5, 0.5, 77)
    v = np.ones(5)
    for expr in ([("main",), ("const", 1.0), ("add",)],                 # X + 1 is dense
                 [("main",), ("exp",)],                                 # exp(0) != 0
                 [("side", 0), ("rowsum",), ("main",), ("mul",)]):      # rowSums of a dense side
        with pytest.raises(ValueError):
            unfused.row_csr(expr, x, [("rowvec", v)], "col")


@pytest.mark.parametrize("seed", range(15))
def test_random_outer_expressions_unfused_equals_interp(seed):
    rng = _rng(4000 + seed)
    m, n, r = int(rng.integers(1, 7)), int(rng.integers(1, 7)), int(rng.integers(1, 6))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = _csr(m, n, 0.5, 4000 + seed)
    u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
    expr = random_scalar_expr(rng, len(kinds), extra_leaf="uvdot")
    for agg in ("none", "full"):
        np.testing.assert_allclose(unfused.outer(expr, x, u, v, sides, agg),
                                   interp.outer(expr, x.rowptr, x.colidx, x.vals, x.shape, u, v, sides, agg),
                                   rtol=1e-11, atol=1e-12, equal_nan=True)


# ------------------------------------------------ plans == generic evaluators ---

def test_workload_plans_equal_generic_unfused_evaluation():
    for name, scale in (("cell", 0.05), ("magg", 0.0005), ("row_dense", 0.0005), ("row_csr", 0.00005), ("outer", 0.01)):
        w = W.make_workload(name, scale)
        if name == "cell":
            a = plans.cell_sum_xyz(w["X"], w["sides"][0][1], w["sides"][1][1])
            b = unfused.cell(w["expr"], w["X"], w["sides"], w["agg"])
        elif name == "magg":
            a = plans.magg_xy_xz_xx(w["X"], w["sides"][0][1], w["sides"][1][1])
            b = unfused.magg(w["exprs"], w["X"], w["sides"])
        elif name == "row_dense":
            a = plans.row_tx_w_xv(w["X"], w["sides"][0][1], w["sides"][1][1])
            b = unfused.row_dense(w["expr"], w["X"], w["sides"], w["agg"])
        elif name == "row_csr":
            x = ops.make_csr(*w["X"])
            a = plans.row_csr_tx_xv(x, w["sides"][0][1])
            b = unfused.row_csr(w["expr"], x, w["sides"], w["agg"])
        else:
            x = ops.make_csr(*w["X"])
            a = plans.outer_sum_x_log_uv(x, w["U"], w["V"])
            b = unfused.outer(w["expr"], x, w["U"], w["V"], w["sides"], w["agg"])
        scale_ = np.abs(a).max() if a.size else 1.0
        assert np.abs(a - b).max() <= 1e-13 * scale_, name


# ---------------------------------------------------- Outer right_mm / left_mm ---

ALS_W = [("main",), ("neq0",), ("uvdot",), ("mul",)]        # (X != 0) * (U_i . V_j), Sec. 2.2 Outer listing


def test_outer_mm_variants_closed_form_dense_formula_and_interp():
    m, n, r = 17, 13, 5
    g = _rng(10)
    u, v = g.uniform(size=(m, r)), g.uniform(size=(n, r))
    x = _csr(m, n, 0.3, 33)
    d = ops.csr_to_dense(x)
    # the ALS-CG update of Sec. 2.2 (first expression): ((X != 0) * (U t(V))) V, and its mirror image
    ref_r = ((d != 0) * (u @ v.T)) @ v
    ref_l = ((d != 0) * (u @ v.T)).T @ u
    np.testing.assert_allclose(unfused.outer(ALS_W, x, u, v, [], "right_mm"), ref_r, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(unfused.outer(ALS_W, x, u, v, [], "left_mm"), ref_l, rtol=1e-12, atol=1e-13)
    for agg in ("right_mm", "left_mm"):
        np.testing.assert_allclose(unfused.outer(ALS_W, x, u, v, [], agg),
                                   interp.outer(ALS_W, x.rowptr, x.colidx, x.vals, x.shape, u, v, [], agg),
                                   rtol=1e-12, atol=1e-13)
    # closed form: U = V = ones, body = X  ->  right: rowSums(X) in every column; left: colSums(X)
    ones_u, ones_v = np.ones((m, r)), np.ones((n, r))
    got = unfused.outer([("main",)], x, ones_u, ones_v, [], "right_mm")
    np.testing.assert_allclose(got, np.repeat(d.sum(1)[:, None], r, 1), rtol=1e-14)
    got = unfused.outer([("main",)], x, ones_u, ones_v, [], "left_mm")
    np.testing.assert_allclose(got, np.repeat(d.sum(0)[:, None], r, 1), rtol=1e-14)
    # rows / columns without stored cells give zero rows
    empty = ops.make_csr(np.zeros(m + 1, np.int64), np.zeros(0, np.int32), np.zeros(0), (m, n))
    assert not unfused.outer(ALS_W, empty, u, v, [], "right_mm").any()
    assert unfused.outer(ALS_W, empty, u, v, [], "left_mm").shape == (n, r)


@pytest.mark.parametrize("seed", range(8))
def test_random_outer_mm_expressions_unfused_equals_interp(seed):
    rng = _rng(4500 + seed)
    m, n, r = int(rng.integers(1, 7)), int(rng.integers(1, 7)), int(rng.integers(1, 5))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = _csr(m, n, 0.5, 4500 + seed)
    u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
    expr = random_scalar_expr(rng, len(kinds), extra_leaf="uvdot")
    for agg in ("right_mm", "left_mm"):
        np.testing.assert_allclose(unfused.outer(expr, x, u, v, sides, agg),
                                   interp.outer(expr, x.rowptr, x.colidx, x.vals, x.shape, u, v, sides, agg),
                                   rtol=1e-11, atol=1e-12, equal_nan=True)


# ----------------------------------------------------- Cell / MAgg over sparse X ---

@pytest.mark.parametrize("seed", range(12))
def test_sparse_cell_equals_dense_cell_on_the_densified_input(seed):
    """Sparse-safe bodies: restricting the evaluation to the stored cells of X does not
    change any aggregate (Sec. 1: sparse drivers), checked against the dense Cell evaluators."""
    rng = _rng(5000 + seed)
    m, n = int(rng.integers(1, 8)), int(rng.integers(1, 9))
    kinds = ["matrix", "colvec", "rowvec", "scalar"]
    sides = _sides(rng, kinds, m, n)
    x = _csr(m, n, 0.4, 5000 + seed)
    d = ops.csr_to_dense(x)
    expr = random_row_expr(rng, kinds, depth=3, want="V", sparse_safe=True, reductions=False)
    for agg in ("full", "row", "col"):
        got = unfused.cell_csr(expr, x, sides, agg)
        np.testing.assert_allclose(got, unfused.cell(expr, d, sides, agg), rtol=1e-11, atol=1e-12, equal_nan=True)
        np.testing.assert_allclose(got, interp.cell(expr, d, sides, agg), rtol=1e-11, atol=1e-12, equal_nan=True)
    got = np.zeros((m, n))
    got[ops.csr_row_index(x), x.colidx] = unfused.cell_csr(expr, x, sides, "none")
    np.testing.assert_allclose(got, unfused.cell(expr, d, sides, "none"), rtol=1e-12, atol=1e-13, equal_nan=True)


def test_sparse_magg_closed_form_and_dense_equivalence():
    m, n = 40, 30
    x = _csr(m, n, 0.1, 71)
    r = _rng(72)
    y, z = r.uniform(-1, 1, size=(2, m, n))
    exprs = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)], [("main",), ("pow2",)]]
    sides = [("matrix", y), ("matrix", z)]
    got = unfused.magg_csr(exprs, x, sides)
    np.testing.assert_allclose(got, plans.magg_xy_xz_xx(ops.csr_to_dense(x), y, z), rtol=1e-13)
    rows = ops.csr_row_index(x)
    ref = [math.fsum(x.vals * y[rows, x.colidx]), math.fsum(x.vals * z[rows, x.colidx]), math.fsum(x.vals ** 2)]
    np.testing.assert_allclose(got, ref, rtol=1e-14)
    with pytest.raises(ValueError):
        unfused.cell_csr([("main",), ("const", 1.0), ("add",)], x, sides, "full")
    with pytest.raises(ValueError):
        unfused.cell_csr([("main",), ("rowsum",)], x, sides, "full")


# ------------------------------------------- Row with a matrix right-hand side ---

MLOG_Q = [("side", 1), ("main",), ("side", 0), ("matmult",), ("mul",)]                   # Q = P * (X V)
MLOGREG = [("main",)] + MLOG_Q + [("side", 1)] + MLOG_Q + [("rowsum",), ("mul",), ("sub",), ("outerk",)]
TXXV = [("main",), ("main",), ("side", 0), ("matmult",), ("outerk",)]                     # t(X) (X V)


def test_row_matrix_rhs_plans_numpy_interp_and_reductions():
    r = _rng(11)
    m, n, k = 60, 9, 4
    x, v, p = r.normal(size=(m, n)), r.normal(size=(n, k)), r.uniform(size=(m, k))
    sides = [("rhs", v), ("kvec", p)]
    ref = x.T @ (x @ v)
    np.testing.assert_allclose(plans.row_tx_xv_matrix(x, v), ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(unfused.row_dense(TXXV, x, sides, "col_t"), ref, rtol=1e-12, atol=1e-12)
    q = p * (x @ v)
    ref2 = x.T @ (q - p * q.sum(1, keepdims=True))
    np.testing.assert_allclose(plans.mlogreg_core(x, v, p), ref2, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(unfused.row_dense(MLOGREG, x, sides, "col_t"), plans.mlogreg_core(x, v, p), rtol=1e-13, atol=1e-13)
    xs, ps = x[:6], p[:6]
    for expr in (TXXV, MLOGREG):
        np.testing.assert_allclose(unfused.row_dense(expr, xs, [("rhs", v), ("kvec", ps)], "col_t"),
                                   interp.row(expr, xs, [("rhs", v), ("kvec", ps)], "col_t"), rtol=1e-12, atol=1e-13)
    # k = 1 reduces to the matrix-vector chain of the Row workload
    np.testing.assert_allclose(unfused.row_dense(TXXV, x, [("rhs", v[:, :1])], "col_t").ravel(),
                               plans.row_tx_w_xv(x, v[:, 0], np.ones(m)), rtol=1e-13, atol=1e-13)
    # k-vector results: X V itself, its column sums, its total, rowSums(Q) per row
    xv = [("main",), ("side", 0), ("matmult",)]
    np.testing.assert_allclose(unfused.row_dense(xv, x, sides, "none"), x @ v, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(unfused.row_dense(xv, x, sides, "col"), (x @ v).sum(0), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(unfused.row_dense(xv, x, sides, "full"), [(x @ v).sum()], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(unfused.row_dense(MLOG_Q + [("rowsum",)], x, sides, "none"), q.sum(1), rtol=1e-12, atol=1e-13)
    for agg in ("none", "col", "full"):
        np.testing.assert_allclose(unfused.row_dense(xv, xs, sides[:1], agg), interp.row(xv, xs, sides[:1], agg), rtol=1e-12, atol=1e-13)
    # ill-formed programs
    for bad in ([("main",), ("side", 1), ("mul",)],                      # row vector (n) times k-vector
                [("side", 0), ("abs",)],                                 # element-wise on the right-hand side
                TXXV + [("abs",)],                                       # outerk must be last
                [("side", 1), ("side", 0), ("matmult",)]):               # k-vector times right-hand side
        with pytest.raises(ValueError):
            unfused.row_dense(bad, x, sides, "col_t")
    with pytest.raises(ValueError):
        unfused.row_dense(TXXV, x, sides, "full")


@pytest.mark.parametrize("seed", range(4))
def test_row_csr_matrix_rhs_equals_dense_semantics_scipy_and_interp(seed):
    """Row bodies with a right-hand side over a CSR main input (vectMatMult / vectOuterMultAdd over the
    stored cells of a row): the same values as the dense evaluator on the densified matrix, as scipy's
    sparse products, and as the per-row interpreter; empty rows and columns give exact zeros."""
    import scipy.sparse as sp
    r = _rng(300 + seed)
    m, n, k = [(40, 13, 3), (7, 50, 1), (64, 9, 5), (25, 25, 16)][seed]
    rp, ci, va = W.csr_bernoulli(m, n, [0.2, 0.1, 0.5, 0.05][seed], 300 + seed)
    x = ops.make_csr(rp, ci, va, (m, n))
    xd = ops.csr_to_dense(x)
    xs = sp.csr_matrix((va, ci, rp), shape=(m, n))
    v, p = r.normal(size=(n, k)), r.uniform(size=(m, k))
    sides = [("rhs", v), ("kvec", p)]
    got = unfused.row_csr(TXXV, x, sides, "col_t")
    np.testing.assert_allclose(got, (xs.T @ (xs @ v)), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got, unfused.row_dense(TXXV, xd, sides, "col_t"), rtol=1e-13, atol=1e-14)
    q = p * (xs @ v)
    np.testing.assert_allclose(unfused.row_csr(MLOGREG, x, sides, "col_t"), xs.T @ (q - p * q.sum(1, keepdims=True)),
                               rtol=1e-11, atol=1e-12)
    for expr in (TXXV, MLOGREG):
        np.testing.assert_allclose(unfused.row_csr(expr, x, sides, "col_t"),
                                   interp.row_sparse(expr, rp, ci, va, (m, n), sides, "col_t"), rtol=1e-11, atol=1e-12)
    xv = [("main",), ("side", 0), ("matmult",)]
    np.testing.assert_allclose(unfused.row_csr(xv, x, sides, "none"), xs @ v, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(unfused.row_csr(xv, x, sides, "col"), (xs @ v).sum(0), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(unfused.row_csr(xv, x, sides, "full"), [(xs @ v).sum()], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(unfused.row_csr(MLOG_Q + [("rowsum",)], x, sides, "none"), q.sum(1), rtol=1e-12, atol=1e-13)
    # rows without stored cells: X V is exactly zero there; columns without stored cells: zero rows of t(X)(XV)
    empty_rows = np.diff(rp) == 0
    assert not unfused.row_csr(xv, x, sides, "none")[empty_rows].any()
    empty_cols = np.bincount(ci, minlength=n) == 0
    assert not got[empty_cols].any()
    # not sparse-safe: the row-vector operand must be zero where X has no stored cell
    for bad in ([("side", 2), ("side", 0), ("matmult",)],                              # dense row vector times V
                [("main",), ("const", 1.0), ("add",), ("side", 0), ("matmult",)],      # (X + 1) V
                [("side", 2), ("main",), ("side", 0), ("matmult",), ("outerk",)]):     # t(dense) (X V)
        with pytest.raises(ValueError):
            unfused.row_csr(bad, x, sides + [("rowvec", np.ones(n))], "col_t")
