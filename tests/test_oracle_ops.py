"""Pins for the basic operators of the CPU oracle (no GPU).

Each operator is checked against something other than itself: exact integer
results, math.fsum brute force, numpy / scipy library routines.
"""
import math
import os
import subprocess
import sys

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ops
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _rng(s):
    return np.random.default_rng(s)


def test_sum_full_exact_and_cancellation():
    assert ops.sum_full(np.arange(1, 100001, dtype=np.float64)) == 100000 * 100001 / 2
    # a plain fp64 running sum returns 0 here; the extended accumulator must not
    assert ops.sum_full(np.array([1e16, 1.0, -1e16])) == 1.0
    assert ops.sum_full(np.zeros(0)) == 0.0


@pytest.mark.parametrize("n", [1, 7, 65535, 65536, 65537, 300001])
def test_sum_full_matches_fsum(n):
    a = _rng(n).uniform(-1, 1, n)
    ref = math.fsum(a.tolist())
    assert abs(ops.sum_full(a) - ref) <= 2 * np.spacing(abs(ref)) + 1e-300


def test_sum_is_thread_count_independent():
    code = ("import numpy as np, sys; sys.path.insert(0, %r); from oracle import ops;"
            "a=np.random.default_rng(3).uniform(-1,1,1000003); print(repr(ops.sum_full(a)), ops.threads())" % ROOT)
    outs = []
    for t in ("1", "3", "8"):
        env = dict(os.environ, OMP_NUM_THREADS=t)
        o = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, check=True)
        val, thr = o.stdout.split()
        assert thr == t
        outs.append(val)
    assert len(set(outs)) == 1


def test_row_and_col_sums_vs_fsum():
    a = _rng(1).normal(size=(37, 53))
    np.testing.assert_allclose(ops.row_sums(a), [math.fsum(r) for r in a.tolist()], rtol=0, atol=1e-14)
    np.testing.assert_allclose(ops.col_sums(a), [math.fsum(c) for c in a.T.tolist()], rtol=0, atol=1e-14)
    # a transposed / strided view must give the sums of the view, not of the buffer
    np.testing.assert_allclose(ops.row_sums(a.T), ops.col_sums(a), rtol=0, atol=0)
    np.testing.assert_allclose(ops.row_sums(a[:, :20]), [math.fsum(r[:20]) for r in a.tolist()], atol=1e-14)


def test_matvec_and_t_matvec():
    r = _rng(2)
    x, v, q = r.normal(size=(41, 29)), r.normal(size=29), r.normal(size=41)
    ref = [math.fsum(x[i, j] * v[j] for j in range(29)) for i in range(41)]
    np.testing.assert_allclose(ops.matvec(x, v), ref, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(ops.matvec(x, v), x @ v, rtol=1e-12, atol=1e-13)
    reft = [math.fsum(x[i, j] * q[i] for i in range(41)) for j in range(29)]
    np.testing.assert_allclose(ops.t_matvec(x, q), reft, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(ops.t_matvec(x, q), x.T @ q, rtol=1e-12, atol=1e-13)
    # a non-square case catches a transposed operand: shapes would not even match
    assert ops.matvec(x, v).shape == (41,) and ops.t_matvec(x, q).shape == (29,)


def test_csr_products_vs_scipy_and_dense():
    m, n = 300, 70
    rowptr, colidx, vals = W.csr_bernoulli(m, n, 0.08, 11)
    x = ops.make_csr(rowptr, colidx, vals, (m, n))
    s = sp.csr_matrix((vals, colidx, rowptr), shape=(m, n))
    r = _rng(4)
    v, q = r.normal(size=n), r.normal(size=m)
    np.testing.assert_allclose(ops.csr_matvec(x, v), s @ v, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ops.csr_t_matvec(x, q), s.T @ q, rtol=1e-13, atol=1e-14)
    d = ops.csr_to_dense(x)
    np.testing.assert_array_equal(d, s.toarray())
    np.testing.assert_allclose(ops.csr_matvec(x, v), ops.matvec(d, v), rtol=1e-15, atol=1e-16)
    np.testing.assert_allclose(ops.csr_t_matvec(x, q), ops.t_matvec(d, q), rtol=1e-15, atol=1e-16)
    a = r.normal(size=vals.size)
    sa = sp.csr_matrix((a, colidx, rowptr), shape=(m, n))
    np.testing.assert_allclose(ops.csr_row_sums(x, a), np.asarray(sa.sum(axis=1)).ravel(), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ops.csr_col_sums(x, a), np.asarray(sa.sum(axis=0)).ravel(), rtol=1e-13, atol=1e-14)
    np.testing.assert_array_equal(ops.csr_row_index(x), s.tocoo().row)


def test_csr_uv_dot_and_matmul_nt():
    m, n, r = 40, 33, 17
    rowptr, colidx, vals = W.csr_bernoulli(m, n, 0.2, 12)
    x = ops.make_csr(rowptr, colidx, vals, (m, n))
    g = _rng(5)
    u, v = g.uniform(size=(m, r)), g.uniform(size=(n, r))
    rows = ops.csr_row_index(x)
    np.testing.assert_allclose(ops.csr_uv_dot(x, u, v), (u[rows] * v[colidx]).sum(1), rtol=1e-14)
    d = ops.matmul_nt(u, v)
    np.testing.assert_allclose(d, u @ v.T, rtol=1e-14)
    np.testing.assert_allclose(ops.csr_uv_dot(x, u, v), d[rows, colidx], rtol=1e-15)
    # brute force for one stored cell
    k = vals.size // 2
    ref = math.fsum(u[rows[k], t] * v[colidx[k], t] for t in range(r))
    assert abs(ops.csr_uv_dot(x, u, v)[k] - ref) <= 2 * np.spacing(ref)
    # leading dimensions: views into wider buffers
    ub, vb = g.uniform(size=(m, r + 5)), g.uniform(size=(n, r + 3))
    np.testing.assert_allclose(ops.csr_uv_dot(x, ub[:, :r], vb[:, :r]),
                               (ub[rows, :r] * vb[colidx, :r]).sum(1), rtol=1e-14)


def test_elementwise_ops_per_element():
    a = np.array([-2.5, -0.0, 0.0, 0.3, 4.0])
    b = np.array([1.5, 2.0, -1.0, 0.3, 0.5])
    assert ops.ew_unary("pow2", a).tolist() == [6.25, 0.0, 0.0, 0.3 * 0.3, 16.0]
    assert ops.ew_unary("neq0", a).tolist() == [1.0, 0.0, 0.0, 1.0, 1.0]
    assert ops.ew_unary("sign", a).tolist() == [-1.0, 0.0, 0.0, 1.0, 1.0]
    assert ops.ew_unary("neg", a).tolist() == [2.5, 0.0, -0.0, -0.3, -4.0]
    assert ops.ew_unary("abs", a).tolist() == [2.5, 0.0, 0.0, 0.3, 4.0]
    np.testing.assert_allclose(ops.ew_unary("log", np.array([1.0, math.e, 100.0])), [0.0, 1.0, math.log(100.0)], rtol=1e-15)
    np.testing.assert_allclose(ops.ew_unary("exp", np.array([0.0, 1.0])), [1.0, math.e], rtol=1e-15)
    np.testing.assert_allclose(ops.ew_unary("sigmoid", np.array([0.0, 2.0])), [0.5, 1 / (1 + math.exp(-2.0))], rtol=1e-15)
    assert ops.ew_binary("sub", a, b).tolist() == [-4.0, -2.0, 1.0, 0.0, 3.5]
    assert ops.ew_binary("div", a, b).tolist() == [-2.5 / 1.5, -0.0, -0.0, 1.0, 8.0]
    assert ops.ew_binary("min", a, b).tolist() == [-2.5, -0.0, -1.0, 0.3, 0.5]
    assert ops.ew_binary("max", a, b).tolist() == [1.5, 2.0, 0.0, 0.3, 4.0]
    assert ops.ew_binary("pow", np.array([2.0, 9.0]), np.array([10.0, 0.5])).tolist() == [1024.0, 3.0]
    assert ops.ew_binary("lt", a, b).tolist() == [1.0, 1.0, 0.0, 0.0, 0.0]
    assert ops.ew_binary("ge", a, b).tolist() == [0.0, 0.0, 1.0, 1.0, 1.0]
    assert ops.ew_binary("eq", a, b).tolist() == [0.0, 0.0, 0.0, 1.0, 0.0]
    assert ops.ew_binary("ne", a, b).tolist() == [1.0, 1.0, 1.0, 0.0, 1.0]
    assert ops.ew_binary("le", a, b).tolist() == [1.0, 1.0, 0.0, 1.0, 0.0]
    assert ops.ew_binary("gt", a, b).tolist() == [0.0, 0.0, 1.0, 0.0, 1.0]
    # outputs are fresh arrays (materialised intermediates), inputs untouched
    c = ops.ew_binary("add", a, 0.0)
    assert c is not a and not np.shares_memory(c, a)


def test_csr_matmul_dense_both_sides_vs_scipy_and_brute_force():
    m, n, r = 37, 29, 6
    rowptr, colidx, vals = W.csr_bernoulli(m, n, 0.25, 13)
    x = ops.make_csr(rowptr, colidx, vals, (m, n))
    g = _rng(6)
    w = g.normal(size=vals.size)
    bv, bu = g.normal(size=(n, r)), g.normal(size=(m, r))
    sw = sp.csr_matrix((w, colidx, rowptr), shape=(m, n))
    np.testing.assert_allclose(ops.csr_matmul_dense(x, w, bv), sw @ bv, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ops.csr_t_matmul_dense(x, w, bu), sw.T @ bu, rtol=1e-13, atol=1e-14)
    # non-square shapes would not even match if the operands were swapped
    assert ops.csr_matmul_dense(x, w, bv).shape == (m, r) and ops.csr_t_matmul_dense(x, w, bu).shape == (n, r)
    rows = ops.csr_row_index(x)
    i, t = 5, 3
    ref = math.fsum(w[k] * bv[colidx[k], t] for k in range(vals.size) if rows[k] == i)
    assert abs(ops.csr_matmul_dense(x, w, bv)[i, t] - ref) <= 4 * np.spacing(abs(ref)) + 1e-300
    j = int(colidx[vals.size // 2])
    ref = math.fsum(w[k] * bu[rows[k], t] for k in range(vals.size) if colidx[k] == j)
    assert abs(ops.csr_t_matmul_dense(x, w, bu)[j, t] - ref) <= 4 * np.spacing(abs(ref)) + 1e-300
    # leading dimension of B
    bb = g.normal(size=(n, r + 4))
    np.testing.assert_allclose(ops.csr_matmul_dense(x, w, bb[:, :r]), sw @ bb[:, :r], rtol=1e-13, atol=1e-14)


def test_matmul_and_t_matmul():
    r = _rng(7)
    a, b, q = r.normal(size=(31, 17)), r.normal(size=(17, 4)), r.normal(size=(31, 3))
    np.testing.assert_allclose(ops.matmul(a, b), a @ b, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ops.t_matmul(a, q), a.T @ q, rtol=1e-13, atol=1e-14)
    assert ops.matmul(a, b).shape == (31, 4) and ops.t_matmul(a, q).shape == (17, 3)
    ref = math.fsum(a[5, t] * b[t, 2] for t in range(17))
    assert abs(ops.matmul(a, b)[5, 2] - ref) <= 4 * np.spacing(abs(ref))
    ref = math.fsum(a[i, 9] * q[i, 1] for i in range(31))
    assert abs(ops.t_matmul(a, q)[9, 1] - ref) <= 4 * np.spacing(abs(ref))
    # views with leading dimensions
    ab, bb = r.normal(size=(31, 20)), r.normal(size=(17, 6))
    np.testing.assert_allclose(ops.matmul(ab[:, 2:19], bb[:, 1:5]), ab[:, 2:19] @ bb[:, 1:5], rtol=1e-13, atol=1e-14)
    # a k = 1 right-hand side reduces to the matrix-vector routines
    np.testing.assert_allclose(ops.matmul(a, b[:, :1]).ravel(), ops.matvec(a, b[:, 0]), rtol=0, atol=0)
    np.testing.assert_allclose(ops.t_matmul(a, q[:, :1]).ravel(), ops.t_matvec(a, q[:, 0]), rtol=0, atol=0)
