"""The five workloads: shapes, distributions, expressions (symbolic), variants.

Shapes, sparsities and distributions follow the paper's micro-benchmarks
(Sec. 5.2, Fig. 8: Cell, MAgg, Row dense/sparse, Outer) at the sizes this build
is measured on.  ``scale`` < 1 shrinks the number of rows (and for Outer also
the columns) for tests; everything else is unchanged.

An expression is a symbolic postfix list of tuples, e.g.
``[("main",), ("side", 0), ("mul",)]``.
"""
from .gen import seed_for, dense_uniform, dense_normal, csr_bernoulli

WORKLOADS = ("cell", "magg", "row_dense", "row_csr", "outer")

EPS = 1e-15


def make_workload(name, scale=1.0):
    """Returns a dict describing workload ``name`` with freshly drawn inputs."""
    if name == "cell":        # sum(X * Y * Z), X,Y,Z 1000 x 1000 uniform[0,1)
        m, n = max(1, int(round(1000 * scale))), 1000
        x = dense_uniform(m, n, 0.0, 1.0, seed_for(1, 0))
        y = dense_uniform(m, n, 0.0, 1.0, seed_for(1, 1))
        z = dense_uniform(m, n, 0.0, 1.0, seed_for(1, 2))
        return dict(template="cell", X=x, sides=[("matrix", y), ("matrix", z)], agg="full",
                    expr=[("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)],
                    bytes=3 * 8 * m * n)
    if name == "magg":        # [sum(X*Y), sum(X*Z), sum(X^2)], 100000 x 1000 uniform[-1,1)
        m, n = max(1, int(round(100000 * scale))), 1000
        x = dense_uniform(m, n, -1.0, 1.0, seed_for(2, 0))
        y = dense_uniform(m, n, -1.0, 1.0, seed_for(2, 1))
        z = dense_uniform(m, n, -1.0, 1.0, seed_for(2, 2))
        return dict(template="magg", X=x, sides=[("matrix", y), ("matrix", z)],
                    exprs=[[("main",), ("side", 0), ("mul",)],
                           [("main",), ("side", 1), ("mul",)],
                           [("main",), ("pow2",)]],
                    bytes=3 * 8 * m * n)
    if name == "row_dense":   # t(X) %*% (w * (X %*% v)), X 1e6 x 100 normal
        m, n = max(1, int(round(1000000 * scale))), 100
        x = dense_normal(m, n, seed_for(3, 0))
        v = dense_normal(n, 1, seed_for(3, 1)).reshape(n)
        w = dense_uniform(m, 1, 0.0, 1.0, seed_for(3, 2)).reshape(m)
        return dict(template="row", X=x, sides=[("rowvec", v), ("colvec", w)], agg="col_t",
                    expr=[("main",), ("side", 0), ("dot",), ("side", 1), ("mul",),
                          ("main",), ("mul",)],
                    bytes=8 * m * n + 8 * m + 16 * n)
    if name == "row_csr":     # t(X) %*% (X %*% v), X CSR 1e7 x 1000 density 0.01
        m, n = max(1, int(round(10000000 * scale))), 1000
        rowptr, colidx, vals = csr_bernoulli(m, n, 0.01, seed_for(4, 0))
        v = dense_normal(n, 1, seed_for(4, 1)).reshape(n)
        nnz = int(rowptr[-1])
        return dict(template="row", X=(rowptr, colidx, vals, (m, n)), sides=[("rowvec", v)],
                    agg="col_t",
                    expr=[("main",), ("side", 0), ("dot",), ("main",), ("mul",)],
                    bytes=12 * nnz + 4 * (m + 1) + 16 * n, nnz=nnz)
    if name == "outer":       # sum(X * log(U %*% t(V) + 1e-15)), X CSR 1e5 x 1e5 density 1e-3
        m = n = max(1, int(round(100000 * scale)))
        r = 100
        rowptr, colidx, vals = csr_bernoulli(m, n, 0.001, seed_for(5, 0))
        u = dense_uniform(m, r, 0.0, 1.0, seed_for(5, 1))
        v = dense_uniform(n, r, 0.0, 1.0, seed_for(5, 2))
        nnz = int(rowptr[-1])
        return dict(template="outer", X=(rowptr, colidx, vals, (m, n)), U=u, V=v, sides=[],
                    agg="full",
                    expr=[("main",), ("uvdot",), ("const", EPS), ("add",), ("log",), ("mul",)],
                    bytes=12 * nnz + 8 * r * nnz + 8 * r * m + 4 * (m + 1), nnz=nnz,
                    bytes_compulsory=12 * nnz + 4 * (m + 1) + 8 * r * (m + n))
    raise KeyError(name)
