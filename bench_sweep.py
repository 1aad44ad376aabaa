#!/usr/bin/env python3
"""Timing sweep over the paper's operator micro-benchmarks (Sec. 5.2, Fig. 8a-8h) on one GPU.

Not the graded benchmark (that is bench.py): this walks the sizes of Fig. 8 -- Cell, MAgg and Row
on x * 10^3 matrices for x in {1e3, 1e4, 1e5, 1e6}, dense and with a sparse X (sparsity 0.1), Row
with a 1e3 x 2 right-hand side, Outer on 2e4 x 2e4 with rank 100 over sparsities 1 .. 1e-4 -- and
prints one line per point: median kernel-call time (HIP events on the launch stream), the
algorithmic bytes of the fused operator and the resulting GB/s (stored cells per second for sparse
inputs).  Dense inputs are drawn on the device (torch.rand), sparse patterns by the seeded
generators of workloads/; results are not compared with the oracle here (tests/ does that at
sizes the oracle can handle), only checked to be finite.

Two more groups follow the end-to-end experiments: "classes" is the shape of the class-count
experiment (Sec. 5.4: 1e7 x 100 dense, t(X)(XV) and the multinomial logistic regression core of
Sec. 2.2 for k = 2 .. 16 classes), "narrow" is Row t(X)(Xv) on the narrow dense matrices of Table 2
(1e8 x 10 scaled to 1e7 x 10, and 29 columns as in Airline78), "mnist" the shape of Mnist8m (784
columns, a quarter of the cells stored, 10 classes; 1e6 rows), sparse and dense.  The "classes" points run 25 untimed calls
first: the matrix-unit kernels speed up over the first ~20 calls on an idle device (the paper's
experiments are iterative algorithms that call an operator many times).

    python bench_sweep.py [--only cell,row] [--max-rows 1000000] [--iters 7]
"""
import argparse
import json
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", default="cell,cell_sparse,magg,magg_sparse,row,row_sparse,row_rhs,outer,classes,narrow,mnist")
    ap.add_argument("--max-rows", type=int, default=1_000_000)
    ap.add_argument("--iters", type=int, default=7)
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench_sweep.py needs a GPU")
    import paper_1801_00829_amd as F
    import workloads as W

    only = set(args.only.split(","))
    n = 1000
    rows = [x for x in (1000, 10_000, 100_000, 1_000_000) if x <= args.max_rows]

    def timed(fn, warm=2):
        for _ in range(warm):
            out = fn()
        torch.cuda.synchronize()
        evs = []
        for _ in range(args.iters):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            out = fn()
            b.record()
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        assert bool(torch.isfinite(out).all()), "non-finite result"
        return ts[len(ts) // 2]

    def report(fig, what, shape, us, nbytes, nnz=None):
        rec = {"fig": fig, "op": what, "shape": shape, "us": round(us, 1), "bytes": int(nbytes),
               "GBps": round(nbytes / us / 1e3, 1)}
        if nnz is not None:
            rec["nnz"] = int(nnz)
            rec["Gnnz_per_s"] = round(nnz / us / 1e3, 2)
        print(json.dumps(rec), flush=True)

    def dev_csr(m, ncols, density, seed):
        rp, ci, va = W.csr_bernoulli(m, ncols, density, seed)
        t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda()
        return F.Csr(t(rp, torch.int32), t(ci, torch.int32), t(va, torch.float64), (m, ncols)), int(rp[-1])

    XYZ = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    XY_XZ = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)]]
    TXV = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    TXXV = [("main",), ("main",), ("side", 0), ("matmult",), ("outerk",)]
    LOGUV = [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]

    for m in rows:
        dense = only & {"cell", "magg", "row", "row_rhs", "cell_sparse", "magg_sparse"}
        if dense:
            x = torch.rand(m, n, dtype=torch.float64, device="cuda")
            y = torch.rand(m, n, dtype=torch.float64, device="cuda")
            z = torch.rand(m, n, dtype=torch.float64, device="cuda")
            v = torch.rand(n, dtype=torch.float64, device="cuda")
            sd = [("matrix", y), ("matrix", z)]
        if "cell" in only:
            report("8a", "Cell sum(X*Y*Z) dense", [m, n], timed(lambda: F.fuse_cell(XYZ, x, sd, "full")), 24 * m * n)
        if "magg" in only:
            report("8c", "MAgg sum(X*Y), sum(X*Z) dense", [m, n], timed(lambda: F.fuse_magg(XY_XZ, x, sd)), 24 * m * n)
        if "row" in only:
            report("8e", "Row t(X)(Xv) dense", [m, n], timed(lambda: F.fuse_row(TXV, x, [("rowvec", v)], "col_t")),
                   8 * m * n + 16 * n)
        if "row_rhs" in only:
            vk = torch.rand(n, 2, dtype=torch.float64, device="cuda")
            report("8g", "Row t(X)(XV) dense, V 1e3x2", [m, n],
                   timed(lambda: F.fuse_row(TXXV, x, [("rhs", vk)], "col_t")), 8 * m * n + 32 * n * 2)
        if only & {"cell_sparse", "magg_sparse", "row_sparse"}:
            xs, nnz = dev_csr(m, n, 0.1, 11)
            if "cell_sparse" in only:
                # sparse driver X, dense Y and Z read at the stored positions (8 + 4 + 2*8 bytes per stored cell)
                report("8b", "Cell sum(X*Y*Z), X sparse 0.1", [m, n],
                       timed(lambda: F.fuse_cell_csr(XYZ, xs, sd, "full")), 28 * nnz + 4 * m, nnz)
            if "magg_sparse" in only:
                report("8d", "MAgg sum(X*Y), sum(X*Z), X sparse 0.1", [m, n],
                       timed(lambda: F.fuse_magg_csr(XY_XZ, xs, sd)), 28 * nnz + 4 * m, nnz)
            if "row_sparse" in only:
                report("8f", "Row t(X)(Xv), X sparse 0.1", [m, n],
                       timed(lambda: F.fuse_row(TXV, xs, [("rowvec", v)], "col_t")), 12 * nnz + 4 * m + 16 * n, nnz)
            del xs
        if dense:
            del x, y, z

    if "outer" in only:
        m = nc = 20_000
        r = 100
        u = torch.rand(m, r, dtype=torch.float64, device="cuda")
        v = torch.rand(nc, r, dtype=torch.float64, device="cuda")
        for sp in (1.0, 0.1, 0.01, 0.001, 0.0001):
            if sp == 1.0:      # all cells stored
                rp = (torch.arange(m + 1, dtype=torch.int64, device="cuda") * nc).to(torch.int32)
                ci = torch.arange(nc, dtype=torch.int32, device="cuda").repeat(m)
                xs, nnz = F.Csr(rp, ci, torch.rand(m * nc, dtype=torch.float64, device="cuda"), (m, nc)), m * nc
            else:
                xs, nnz = dev_csr(m, nc, sp, 13)
            us = timed(lambda: F.fuse_outer(LOGUV, xs, u, v, [], "full"))
            report("8h", "Outer sum(X*log(U t(V)+1e-15)) sparsity %g" % sp, [m, nc, r], us,
                   12 * nnz + 8 * r * nnz + 8 * r * m, nnz)
            del xs

    if "narrow" in only:
        for (m, nc) in ((10_000_000, 10), (14_000_000, 29)):
            x = torch.randn(m, nc, dtype=torch.float64, device="cuda")
            v = torch.randn(nc, dtype=torch.float64, device="cuda")
            report("tab2", "Row t(X)(Xv) dense, narrow", [m, nc],
                   timed(lambda: F.fuse_row(TXV, x, [("rowvec", v)], "col_t")), 8 * m * nc + 16 * nc)
            del x

    if "mnist" in only:
        # the shape of Mnist8m (Table 2: 784 columns, a quarter of the cells stored, 10 classes), 1e6 rows
        m, nc, k = 1_000_000, 784, 10
        q = [("side", 1), ("main",), ("side", 0), ("matmult",), ("mul",)]
        mlogreg = [("main",)] + q + [("side", 1)] + q + [("rowsum",), ("mul",), ("sub",), ("outerk",)]
        xs, nnz = dev_csr(m, nc, 0.25, 17)
        vk = torch.randn(nc, k, dtype=torch.float64, device="cuda")
        p = torch.rand(m, k, dtype=torch.float64, device="cuda")
        report("tab2", "Row t(X)(XV), X sparse 0.25, k=10", [m, nc],
               timed(lambda: F.fuse_row(TXXV, xs, [("rhs", vk)], "col_t"), warm=10), 12 * nnz + 4 * m, nnz)
        report("tab2", "Row t(X)(Q - P*rowSums(Q)), Q = P*(XV), X sparse 0.25, k=10", [m, nc],
               timed(lambda: F.fuse_row(mlogreg, xs, [("rhs", vk), ("kvec", p)], "col_t"), warm=10),
               12 * nnz + 4 * m + 8 * m * k, nnz)
        xd = torch.randn(m, nc, dtype=torch.float64, device="cuda")
        report("tab2", "Row t(X)(XV) dense, k=10", [m, nc],
               timed(lambda: F.fuse_row(TXXV, xd, [("rhs", vk)], "col_t"), warm=10), 8 * m * nc)
        report("tab2", "Row t(X)(Q - P*rowSums(Q)), Q = P*(XV) dense, k=10", [m, nc],
               timed(lambda: F.fuse_row(mlogreg, xd, [("rhs", vk), ("kvec", p)], "col_t"), warm=10), 8 * m * nc + 8 * m * k)
        del xs, xd, p

    if "classes" in only:
        m, nc = 10_000_000, 100
        q = [("side", 1), ("main",), ("side", 0), ("matmult",), ("mul",)]
        mlogreg = [("main",)] + q + [("side", 1)] + q + [("rowsum",), ("mul",), ("sub",), ("outerk",)]
        x = torch.randn(m, nc, dtype=torch.float64, device="cuda")
        for k in (2, 4, 8, 16):
            vk = torch.randn(nc, k, dtype=torch.float64, device="cuda")
            p = torch.rand(m, k, dtype=torch.float64, device="cuda")
            report("sec5.4", "Row t(X)(XV) dense, k=%d" % k, [m, nc],
                   timed(lambda: F.fuse_row(TXXV, x, [("rhs", vk)], "col_t"), warm=25), 8 * m * nc + 16 * nc * k)
            report("sec5.4", "Row t(X)(Q - P*rowSums(Q)), Q = P*(XV), k=%d" % k, [m, nc],
                   timed(lambda: F.fuse_row(mlogreg, x, [("rhs", vk), ("kvec", p)], "col_t"), warm=25),
                   8 * m * nc + 8 * m * k + 16 * nc * k)
            del p
        del x


if __name__ == "__main__":
    main()
