"""The five benchmark workloads as explicit unfused plans -- TEST INFRASTRUCTURE ONLY.

Each function is the chain of basic operators that the paper's fused operator
replaces, written out step by step (every arrow of the plan is one call into
``oracle.ops`` that materialises its output).
"""
import numpy as np

from . import ops


def cell_sum_xyz(x, y, z):
    """sum(X * Y * Z), Fig. 1a: two materialised intermediates, then the sum."""
    t1 = ops.ew_binary("mul", x, y)
    t2 = ops.ew_binary("mul", t1, z)
    return np.array([ops.sum_full(t2)])


def magg_xy_xz_xx(x, y, z):
    """[sum(X*Y), sum(X*Z), sum(X^2)]: three aggregates, each evaluated on its
    own (Sec. 5.2 "Multi-Aggregate Operations": per-aggregate operators re-read X)."""
    s1 = ops.sum_full(ops.ew_binary("mul", x, y))
    s2 = ops.sum_full(ops.ew_binary("mul", x, z))
    s3 = ops.sum_full(ops.ew_unary("pow2", x))
    return np.array([s1, s2, s3])


def row_tx_w_xv(x, v, w):
    """t(X) %*% (w * (X %*% v)), Fig. 1b with a weight vector: matrix-vector
    product, element-wise scale, then a second scan of X for the transposed product."""
    q = ops.matvec(x, v)
    q2 = ops.ew_binary("mul", w, q)
    return ops.t_matvec(x, q2)


def row_csr_tx_xv(x: ops.Csr, v):
    """t(X) %*% (X %*% v) for CSR X (Sec. 5.2 "Row Operations", sparse)."""
    q = ops.csr_matvec(x, v)
    return ops.csr_t_matvec(x, q)


def outer_sum_x_log_uv(x: ops.Csr, u, v, eps=1e-15):
    """sum(X * log(U %*% t(V) + eps)), Fig. 1d, restricted to the stored cells
    of X (the multiply with X is the sparse driver): per stored cell the inner
    product, then + eps, log, multiply by the cell's value, and the sum."""
    p = ops.csr_uv_dot(x, u, v)
    p1 = ops.ew_binary("add", p, eps)
    p2 = ops.ew_unary("log", p1)
    p3 = ops.ew_binary("mul", x.vals, p2)
    return np.array([ops.sum_full(p3)])


def outer_sum_x_log_uv_dense(x_dense, u, v, eps=1e-15):
    """The literal dense plan of Fig. 1d (tiny inputs only): materialise
    U %*% t(V), add eps, take the log of every cell, multiply by X, sum."""
    d = ops.matmul_nt(u, v)
    d1 = ops.ew_binary("add", d, eps)
    d2 = ops.ew_unary("log", d1)
    d3 = ops.ew_binary("mul", x_dense, d2)
    return np.array([ops.sum_full(d3)])


def row_tx_xv_matrix(x, v):
    """t(X) %*% (X %*% V) with an n x k right-hand side (Fig. 8g): two matrix products."""
    return ops.t_matmul(x, ops.matmul(x, v))


def mlogreg_core(x, v, p):
    """The inner-loop core of multinomial logistic regression (Sec. 2.2, second example):
    Q = P * (X %*% V);  H = t(X) %*% (Q - P * rowSums(Q)), operator by operator."""
    xv = ops.matmul(x, v)
    q = ops.ew_binary("mul", p, xv)
    rs = ops.row_sums(q).reshape(-1, 1)
    t1 = ops.ew_binary("mul", p, rs)
    t2 = ops.ew_binary("sub", q, t1)
    return ops.t_matmul(x, t2)
