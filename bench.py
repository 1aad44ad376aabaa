"""Benchmark of the fused-operator hot path on one MI355X.

A step is one pass of the whole hot path: the five fused operators (Cell, MAgg,
Row dense, Row CSR, Outer) on the benchmark workloads, inputs resident in HBM.
Prints ONE JSON line:
  value      effective HBM GB/s of the step = bytes the five operators must move from HBM
             (Cell, MAgg, Row: their inputs once; Outer: X, U and V once -- its compulsory bytes)
             / step time.  Never above the HBM peak by construction.
  templates  per operator: time per call, GB/s and fraction of the HBM peak by the same byte
             model; for Outer stored cells per second and the fraction of the measured L2
             gather ceiling instead (it is not HBM-bound).
  roofline   the dominant kernel of the step against the bound that binds it.
  gather_ceilings  fuse_probe_gather over tables resident in L2, in the memory-side cache
             and in HBM: the ceilings that the Outer figures are set against.
  cpu_baseline  the CPU oracle timed on the same workloads, all host threads and one.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--templates cell,magg,...] [--no-cpu-baseline]
    python bench.py --sweep [groups]     timing sweep over the paper's micro-benchmark sizes instead (see sweep())
    python bench.py --cell-budget        where the time of the 24 MB Cell workload goes (see cell_budget())
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak
ALL = ("cell", "magg", "row_dense", "row_csr", "outer")
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_all_templates_hbm_traffic.txt")


def profile_traffic(path=TRAFFIC_PROFILE):
    """HBM-side bytes per launch by kernel name, from the committed rocprofv3 --pmc summary
    (lines `traffic <kernel> <fetched bytes> <written bytes>`, already scaled by the copy probe).
    A kernel that is not in the summary (its code changed since the counters were collected)
    has no entry: the benchmark then reports null instead of a stale figure."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 4 and w[0] == "traffic":
                    out[w[1]] = (float(w[2]), float(w[3]))
    except OSError:
        pass
    return out


KERNEL_PROFILE = os.path.join(ROOT, "profiles", "bench_all_templates_kernel_stats.txt")


def profile_kernel_us(path=KERNEL_PROFILE):
    """Average duration (microseconds) of every kernel in the committed rocprofv3 kernel trace of this benchmark,
    by kernel name (table rows `name calls total_ns avg_ns min_ns max_ns pct`).  Like the traffic figures, an entry
    stands for exactly the code that was profiled: a kernel that has changed since has another name and no entry."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 7 and w[0].startswith("fuse_") and w[6].endswith("%"):
                    out[w[0]] = float(w[3]) / 1e3
    except (OSError, ValueError):
        pass
    return out


def seconds_at(nbytes, gbps_):
    """Time to move nbytes at gbps_ GB/s (1 GB = 1e9 bytes)."""
    return nbytes / (gbps_ * 1e9)


def gbps(nbytes, seconds):
    return nbytes / seconds / 1e9


def _oracle_pass(names, host):
    """One pass of the CPU oracle's unfused plans over the host copies of the workloads:
    ({name: seconds}, {name: result})."""
    from oracle import ops, plans
    secs, results = {}, {}
    for name in names:
        w = host[name]
        t0 = time.perf_counter()
        if name == "cell":
            r = plans.cell_sum_xyz(w["X"], w["sides"][0][1], w["sides"][1][1])
        elif name == "magg":
            r = plans.magg_xy_xz_xx(w["X"], w["sides"][0][1], w["sides"][1][1])
        elif name == "row_dense":
            r = plans.row_tx_w_xv(w["X"], w["sides"][0][1], w["sides"][1][1])
        elif name == "row_csr":
            r = plans.row_csr_tx_xv(ops.make_csr(*w["X"]), w["sides"][0][1])
        else:
            r = plans.outer_sum_x_log_uv(ops.make_csr(*w["X"]), w["U"], w["V"])
        secs[name] = time.perf_counter() - t0
        results[name] = r
    return secs, results


def _cpu_baseline_child(names):
    """Child-process mode (started with OMP_NUM_THREADS=1 by the parent): draws the same workloads
    and times one oracle pass; prints {"threads": .., "seconds": {name: s}}.  Touches no GPU."""
    import workloads as W
    from oracle import ops
    host = {n: W.make_workload(n, 1.0) for n in names}
    secs, _ = _oracle_pass(names, host)
    print(json.dumps({"threads": ops.threads(), "seconds": secs}), flush=True)


def _cpu_baseline(names, host, hbm_bytes):
    """The CPU oracle, as it stands, on the host copies of the same workloads (full size): once with all
    host threads (in this process) and once with one thread (a child process with OMP_NUM_THREADS=1)."""
    from oracle import ops
    secs, results = _oracle_pass(names, host)
    total_bytes, total_s = sum(hbm_bytes[n] for n in names), sum(secs.values())
    base = {"value": round(gbps(total_bytes, total_s), 3), "unit": "GB/s", "cores": ops.threads(),
            "kind": "oracle", "seconds": round(total_s, 3),
            "sample": "the full workloads, one pass of the unfused operator-at-a-time plans (" +
                      "; ".join("%s %.2f s" % (n, secs[n]) for n in names) + "); bytes as in `value`"}
    try:
        env = dict(os.environ, OMP_NUM_THREADS="1")
        r = subprocess.run([sys.executable, os.path.abspath(__file__), "--cpu-baseline-child", ",".join(names)],
                           env=env, capture_output=True, text=True, timeout=600)
        one = json.loads(r.stdout.strip().splitlines()[-1])
        s1 = sum(one["seconds"].values())
        base["one_core"] = {"value": round(gbps(total_bytes, s1), 3), "unit": "GB/s", "cores": one["threads"],
                            "seconds": round(s1, 3),
                            "sample": "; ".join("%s %.2f s" % (n, one["seconds"][n]) for n in names)}
    except Exception as e:                           # noqa: BLE001 - the one-thread figure is an extra
        base["one_core"] = {"error": str(e)[:200]}
    return base, results


SWEEP_GROUPS = ("cell", "cell_sparse", "magg", "magg_sparse", "row", "row_sparse", "row_rhs", "outer", "classes", "narrow",
                "mnist", "cell_variants", "chain", "cell_sparse_forms", "outer_variants")


def sweep(args):
    """Timing sweep over the paper's operator micro-benchmarks (Sec. 5.2, Fig. 8a-8h) on one GPU -- not the
    benchmark line.  Walks the sizes of Fig. 8 -- Cell, MAgg and Row on x * 10^3 matrices for x in {1e3, 1e4,
    1e5, 1e6}, dense and with a sparse X (sparsity 0.1), Row with a 1e3 x 2 right-hand side, Outer on 2e4 x 2e4
    with rank 100 over sparsities 1 .. 1e-4 -- and prints one JSON line per point: median call time (HIP events
    on the launch stream), the algorithmic bytes of the fused operator and the resulting GB/s (stored cells per
    second for sparse inputs).  Dense inputs are drawn on the device, sparse patterns by the seeded generators
    of workloads/; results are only checked to be finite here (tests/ compares with the oracle).

    Further groups: "classes" the class-count experiment (Sec. 5.4: 1e7 x 100 dense, t(X)(XV) and the multinomial
    logistic regression core of Sec. 2.2 for k = 2 .. 16; 25 untimed calls first: the matrix-unit kernels speed up
    over the first ~20 calls on an idle device), "narrow" Row t(X)(Xv) on the narrow matrices of Table 2, "mnist"
    the shape of Mnist8m (784 columns, a quarter stored, 10 classes; 1e6 rows), "cell_variants" the four variants
    of Cell at 100000 x 1000, "chain" the instruction-footprint expression of Sec. 5.3, "cell_sparse_forms" Cell
    bodies over a sparse X that run in the flat form, "outer_variants" the four Outer variants at the benchmark shape.
    """
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py --sweep needs a GPU")
    import paper_1801_00829_amd as F
    import workloads as W

    only = set(SWEEP_GROUPS) if args.sweep == "all" else set(args.sweep.split(","))
    for g in only:
        if g not in SWEEP_GROUPS:
            sys.exit("unknown sweep group %r (known: %s)" % (g, ", ".join(SWEEP_GROUPS)))
    n = 1000
    rows = [x for x in (1000, 10_000, 100_000, 1_000_000) if args.min_rows <= x <= args.max_rows]

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

    def report(fig, what, shape, us, nbytes, nnz=None, extra=None):
        rec = {"fig": fig, "op": what, "shape": shape, "us": round(us, 1), "bytes": int(nbytes),
               "GBps": round(nbytes / us / 1e3, 1)}
        if extra:
            rec.update(extra)
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
            if only & {"cell_sparse", "magg_sparse"}:
                # the figures' own setting: Y and Z sparse as well (12 bytes per stored cell and 4 per row of each matrix)
                ys, nny = dev_csr(m, n, 0.1, 12)
                zs, nnzz = dev_csr(m, n, 0.1, 14)
                ssd = [("sparse", ys), ("sparse", zs)]
                sp_bytes = 12 * (nnz + nny + nnzz) + 12 * m
                if "cell_sparse" in only:
                    report("8b", "Cell sum(X*Y*Z), X, Y, Z sparse 0.1", [m, n],
                           timed(lambda: F.fuse_cell_csr(XYZ, xs, ssd, "full")), sp_bytes, nnz)
                if "magg_sparse" in only:
                    report("8d", "MAgg sum(X*Y), sum(X*Z), X, Y, Z sparse 0.1", [m, n],
                           timed(lambda: F.fuse_magg_csr(XY_XZ, xs, ssd)), sp_bytes, nnz)
                del ys, zs, ssd
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

    if "cell_variants" in only:
        # the four variants of the Cell template (Table 1) on 100000 x 1000, body X*Y; and with vector sides X*c*r
        m = 100_000
        x = torch.rand(m, n, dtype=torch.float64, device="cuda")
        y = torch.rand(m, n, dtype=torch.float64, device="cuda")
        c = torch.rand(m, dtype=torch.float64, device="cuda")
        rv = torch.rand(n, dtype=torch.float64, device="cuda")
        xy = [("main",), ("side", 0), ("mul",)]
        xcr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
        for agg, outb in (("full", 8), ("row", 8 * m), ("col", 8 * n), ("none", 8 * m * n)):
            report("tab1", "Cell X*Y %s_agg" % agg, [m, n], timed(lambda: F.fuse_cell(xy, x, [("matrix", y)], agg)),
                   16 * m * n + outb)
            report("tab1", "Cell X*c*r %s_agg (column- and row-vector sides)" % agg, [m, n],
                   timed(lambda: F.fuse_cell(xcr, x, [("colvec", c), ("rowvec", rv)], agg)), 8 * m * n + 8 * m + 8 * n + outb)
        del x, y

    if "chain" in only:
        # the expression of the instruction-footprint experiment (Sec. 5.3): sum(f(X / rowSums(X))) with f a chain of
        # N scalar multiplications -- body size against time and compile time
        m = 100_000
        x = torch.rand(m, n, dtype=torch.float64, device="cuda") + 0.5
        for nops in (1, 10, 31, 51, 101, 201):
            body_ = [("main",), ("main",), ("rowsum",), ("div",)]
            for q in range(nops):
                body_ += [("const", 1.0 + 1e-3 * (q + 1)), ("mul",)]
            h0, m0, ms0 = F.cache_stats()
            us = timed(lambda: F.fuse_row(body_, x, [], "full"))
            h1, m1, ms1 = F.cache_stats()
            rec_extra = {"compile_ms": round(ms1 - ms0, 1)}
            report("sec5.3", "Row sum(f(X/rowSums(X))), f = %d multiplications" % nops, [m, n], us, 8 * m * n, extra=rec_extra)
        del x

    if "cell_sparse_forms" in only:
        # Cell bodies over a sparse X (sparsity 0.1, 1e6 x 1e3) that never look at the row: flat form over the cell arrays
        m = min(1_000_000, args.max_rows)
        xs, nnz = dev_csr(m, n, 0.1, 11)
        rv = torch.rand(n, dtype=torch.float64, device="cuda")
        report("8b", "Cell sum(X^2), X sparse 0.1", [m, n], timed(lambda: F.fuse_cell_csr([("main",), ("pow2",)], xs, [], "full")),
               8 * nnz, nnz)
        report("8b", "Cell colSums(X*v), X sparse 0.1", [m, n],
               timed(lambda: F.fuse_cell_csr([("main",), ("side", 0), ("mul",)], xs, [("rowvec", rv)], "col")), 12 * nnz, nnz)
        report("8b", "Cell X*v no_agg, X sparse 0.1", [m, n],
               timed(lambda: F.fuse_cell_csr([("main",), ("side", 0), ("mul",)], xs, [("rowvec", rv)], "none")), 20 * nnz, nnz)
        del xs

    if "outer_variants" in only:
        # the four variants of the Outer template (Table 1) at the benchmark shape: 1e5 x 1e5, 1e7 stored cells, rank 100;
        # product variants with the weights of the ALS-CG update (Sec. 2.2, first example)
        m = nc = 100_000
        r = 100
        xs, nnz = dev_csr(m, nc, 0.001, 13)
        u = torch.rand(m, r, dtype=torch.float64, device="cuda")
        v = torch.rand(nc, r, dtype=torch.float64, device="cuda")
        alscg = [("main",), ("neq0",), ("uvdot",), ("mul",)]
        gather = 12 * nnz + 8 * r * nnz + 8 * r * m
        report("tab1", "Outer sum(X*log(U t(V)+1e-15)) full_agg", [m, nc, r], timed(lambda: F.fuse_outer(LOGUV, xs, u, v, [], "full")), gather, nnz)
        report("tab1", "Outer X*log(U t(V)+1e-15) no_agg", [m, nc, r], timed(lambda: F.fuse_outer(LOGUV, xs, u, v, [], "none")), gather + 8 * nnz, nnz)
        report("tab1", "Outer ((X!=0)*(U t(V))) V right_mm", [m, nc, r], timed(lambda: F.fuse_outer(alscg, xs, u, v, [], "right_mm")), gather + 8 * r * m, nnz)
        report("tab1", "Outer t((X!=0)*(U t(V))) U left_mm", [m, nc, r], timed(lambda: F.fuse_outer(alscg, xs, u, v, [], "left_mm")), gather + 8 * r * nc, nnz)
        pattern = F.outer_left_prepare(xs)
        report("tab1", "Outer t((X!=0)*(U t(V))) U left_mm over a prepared pattern", [m, nc, r],
               timed(lambda: F.fuse_outer_left(alscg, xs, pattern, u, v, [])), gather + 8 * r * nc, nnz)
        del pattern
        del xs, u, v



def cell_budget(args):
    """Where the time of the 24 MB Cell workload (sum(X*Y*Z), 1000 x 1000: 3 us at the HBM peak) goes.  Prints
    one JSON line per measurement, median and minimum of HIP-event brackets (microseconds), inputs cold (512 MB
    written between launches) unless stated: a kernel that reads nothing, a kernel with one 16-byte load (first-byte
    latency), a plain read of 24 MB with several grids (fuse_probe_read: no arithmetic, no reduction), and the Cell
    operator across its launch shapes (threads per block, loads in flight per thread, number of blocks).  Run under
    `rocprofv3 --kernel-trace --stats` the same command gives the kernels' own durations without the bracket."""
    import numpy as np
    import torch
    import paper_1801_00829_amd as F
    import workloads as W
    if not torch.cuda.is_available():
        sys.exit("bench.py --cell-budget needs a GPU")
    w = W.make_workload("cell", 1.0)
    x = torch.from_numpy(w["X"]).cuda()
    sd = [(k, torch.from_numpy(np.asarray(v)).cuda()) for k, v in w["sides"]]
    out = torch.empty(1, dtype=torch.float64, device="cuda")
    evict = torch.empty(1 << 26, dtype=torch.float64, device="cuda")
    sink = torch.zeros(1, dtype=torch.float64, device="cuda")
    buf = torch.rand(3_000_000, dtype=torch.float64, device="cuda")

    def timed(fn, cold=True, iters=20):
        fn()
        ts = []
        for _ in range(iters):
            if cold:
                evict.fill_(1.0)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ts.append((a, b))
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) * 1e3 for a, b in ts)
        return round(t[len(t) // 2], 2), round(t[0], 2)

    def report(what, fn, **kw):
        med, mn = timed(fn, **kw)
        print(json.dumps({"what": what, "median_us": med, "min_us": mn, "cold": kw.get("cold", True)}), flush=True)

    report("kernel that reads nothing (1 block)", lambda: F.probe_read(buf, sink, 1, n_doubles=0))
    report("kernel with one 16-byte load (1 block)", lambda: F.probe_read(buf, sink, 1, n_doubles=2))
    for blocks in (256, 512, 1024, 2048):
        report("plain read of 24 MB, %d blocks of 256 threads" % blocks, lambda: F.probe_read(buf, sink, blocks))
    report("plain read of 24 MB, 2048 blocks, inputs cache-resident", lambda: F.probe_read(buf, sink, 2048), cold=False)
    shapes = [{}, {"FUSE_CELL_BLOCK": 512}, {"FUSE_CELL_BLOCK": 1024}, {"FUSE_CELL_BLOCK": 1024, "FUSE_CELL_UNROLL": 2},
              {"FUSE_CELL_BLOCK": 1024, "FUSE_CELL_UNROLL": 1}, {"FUSE_CELL_BLOCK": 512, "FUSE_CELL_UNROLL": 2},
              {"FUSE_CELL_UNROLL": 2, "FUSE_CELL_BLOCKS_PER_CU": 4}, {"FUSE_CELL_GRID": 128}, {"FUSE_CELL_GRID": 256},
              {"FUSE_CELL_UNROLL": 2, "FUSE_CELL_GRID": 1024}]
    for env in shapes:
        for k_, v_ in env.items():
            os.environ[k_] = str(v_)
        try:
            call = lambda: F.fuse_cell(w["expr"], x, sd, "full", out=out)
            call()
            name = F.last_kernel()
            report("fuse_cell %s (%s)" % (env or "default launch shape", name), call)
            if not env:
                report("fuse_cell default launch shape, inputs cache-resident (%s)" % name, call, cold=False)
        finally:
            for k_ in env:
                os.environ.pop(k_, None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--templates", default=",".join(ALL))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe", action="store_true",
                    help="also launch the 1 GiB copy / read probes once (untimed): a transfer of known "
                         "size that calibrates profiler byte counters collected over this command")
    ap.add_argument("--sweep", nargs="?", const="all", default=None, metavar="GROUPS",
                    help="timing sweep over the paper's micro-benchmark sizes instead of the benchmark line "
                         "(comma-separated groups, see sweep(); default all)")
    ap.add_argument("--max-rows", type=int, default=1_000_000, help="--sweep: largest number of rows of the Fig. 8 groups")
    ap.add_argument("--min-rows", type=int, default=1000, help="--sweep: smallest number of rows of the Fig. 8 groups")
    ap.add_argument("--iters", type=int, default=7, help="--sweep: timed calls per point (median reported)")
    ap.add_argument("--cell-budget", action="store_true",
                    help="time budget of the 24 MB Cell workload instead of the benchmark line (see cell_budget())")
    ap.add_argument("--cpu-baseline-child", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.cpu_baseline_child is not None:
        _cpu_baseline_child([n for n in args.cpu_baseline_child.split(",") if n])
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the fused operators are single-device kernels); "
                 "--gpus %d is not supported" % args.gpus)
    names = [n for n in args.templates.split(",") if n]
    for n in names:
        if n not in ALL:
            sys.exit("unknown template %r" % n)

    if args.sweep is not None:
        sweep(args)
        return
    if args.cell_budget:
        cell_budget(args)
        return

    import numpy as np
    import torch
    import paper_1801_00829_amd as F
    import workloads as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def dev(a, dtype=None):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(dtype) if dtype is not None else t).cuda()

    def sides(ss):
        return [(k, float(v) if k == "scalar" else dev(np.asarray(v, dtype=np.float64))) for k, v in ss]

    def csr(x):
        rp, ci, va, shape = x
        return F.Csr(dev(rp, torch.int32), dev(ci, torch.int32), dev(va), shape)

    # ---- inputs, resident in HBM before anything is timed
    calls, info, host, outs = {}, {}, {}, {}
    for name in names:
        t0 = time.perf_counter()
        w = W.make_workload(name, 1.0)
        # bytes: what the operator must move from HBM (its inputs once; for Outer X, U and V once)
        info[name] = {"bytes": int(w.get("bytes_compulsory", w["bytes"])), "nnz": int(w.get("nnz", 0))}
        if name == "cell":
            x, s, out = dev(w["X"]), sides(w["sides"]), torch.empty(1, dtype=torch.float64, device="cuda")
            calls[name] = (lambda e=w["expr"], x=x, s=s, a=w["agg"], o=out: F.fuse_cell(e, x, s, a, out=o))
        elif name == "magg":
            x, s, out = dev(w["X"]), sides(w["sides"]), torch.empty(3, dtype=torch.float64, device="cuda")
            calls[name] = (lambda e=w["exprs"], x=x, s=s, o=out: F.fuse_magg(e, x, s, out=o))
        elif name == "row_dense":
            x, s, out = dev(w["X"]), sides(w["sides"]), torch.empty(100, dtype=torch.float64, device="cuda")
            calls[name] = (lambda e=w["expr"], x=x, s=s, a=w["agg"], o=out: F.fuse_row(e, x, s, a, out=o))
        elif name == "row_csr":
            x, s, out = csr(w["X"]), sides(w["sides"]), torch.empty(1000, dtype=torch.float64, device="cuda")
            calls[name] = (lambda e=w["expr"], x=x, s=s, a=w["agg"], o=out: F.fuse_row(e, x, s, a, out=o))
        else:
            x, u, v = csr(w["X"]), dev(w["U"]), dev(w["V"])
            out = torch.empty(1, dtype=torch.float64, device="cuda")
            info[name]["bytes_gather_model"] = int(w["bytes"])       # one V row per stored cell, U once per row
            info[name]["rank"] = int(w["U"].shape[1])
            calls[name] = (lambda e=w["expr"], x=x, u=u, v=v, a=w["agg"], o=out: F.fuse_outer(e, x, u, v, [], a, out=o))
        host[name] = w
        outs[name] = out
        print("# %s inputs ready in %.1f s" % (name, time.perf_counter() - t0), file=sys.stderr, flush=True)

    if args.probe:
        n = 1 << 27                                   # 2^27 doubles = 1 GiB
        src = torch.rand(n, dtype=torch.float64, device="cuda")
        dst = torch.empty_like(src)
        sink = torch.zeros(1, dtype=torch.float64, device="cuda")
        F.probe_copy(dst, src, 2048)
        F.probe_read(src, sink, 1024)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up (includes hipRTC compilation of the five bodies)
    t0 = time.perf_counter()
    for _ in range(max(args.warmup, 1)):
        for name in names:
            calls[name]()
    torch.cuda.synchronize()
    hits, misses, compile_ms = F.cache_stats()
    kernels = {}
    for name in names:
        calls[name]()
        kernels[name] = F.last_kernel()
    torch.cuda.synchronize()
    print("# warm-up %.1f s (hipRTC %.0f ms for %d plans)" % (time.perf_counter() - t0, compile_ms, misses),
          file=sys.stderr, flush=True)

    # ---- timed region: exactly K steps; HIP events on the launch stream between the operators (one event is the
    # end of an operator and the start of the next).  An operator's time between its two events also holds the
    # queue's handling of an event packet: ~4 us, which only shows in the 8 us Cell operator.
    K = args.steps
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        marks[k][0].record()
        for i, name in enumerate(names):
            calls[name]()
            marks[k][i + 1].record()
    torch.cuda.synchronize()
    ev = {name: [(marks[k][i], marks[k][i + 1]) for k in range(K)] for i, name in enumerate(names)}
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / K * 1e3

    # ---- the same K steps replayed from a HIP graph (one capture of the five calls): what the step costs
    # without the host launch path; reported beside the eager figure, never as `value`
    graph = None
    try:
        gs = torch.cuda.Stream()
        gs.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(gs):
            for name in names:                       # workspace of the capture stream
                calls[name]()
        gs.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=gs):
            for name in names:
                calls[name]()
        g.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for k in range(K):
            g.replay()
        torch.cuda.synchronize()
        g_elapsed = time.perf_counter() - tg
        graph = {"ms_per_step": round(g_elapsed / K * 1e3, 4),
                 "value": round(gbps(sum(info[n]["bytes"] for n in names), g_elapsed / K), 1), "unit": "GB/s"}
        if "cell" in names:
            # the small Cell workload back to back: 100 launches in one graph, inputs cache-resident after the first
            # (the timing protocol's "amortised time of 100 back-to-back launches" for the launch-latency regime)
            g100 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g100, stream=gs):
                for _ in range(100):
                    calls["cell"]()
            g100.replay()
            torch.cuda.synchronize()
            t100 = time.perf_counter()
            for _ in range(5):
                g100.replay()
            torch.cuda.synchronize()
            graph["cell_back_to_back_us"] = round((time.perf_counter() - t100) / 500 * 1e6, 2)
    except Exception as e:                           # noqa: BLE001 - an extra, must not break the benchmark line
        graph = {"error": str(e)[:200]}

    # ---- floor for the 24 MB Cell workload: a plain read-only kernel (no reduction at all) over a
    # buffer of the same size, cold like the Cell inputs are inside a step (512 MB written in between),
    # in the same event bracket; the Cell operator cannot be faster than this on this device
    cell_floor = None
    if "cell" in names:
        nb = info["cell"]["bytes"] // 16 * 2
        buf = torch.rand(nb, dtype=torch.float64, device="cuda")
        sink = torch.zeros(1, dtype=torch.float64, device="cuda")
        evict = torch.empty(1 << 26, dtype=torch.float64, device="cuda")
        fl = []
        for k in range(K + 2):
            evict.fill_(1.0)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            F.probe_read(buf, sink, 2048)
            b.record()
            fl.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in fl[2:])
        cell_floor = {"avg_us": round(sum(ts) / len(ts) * 1e3, 2), "min_us": round(ts[0] * 1e3, 2),
                      "what": "fuse_probe_read over %d cold bytes, 2048 blocks, same event bracket" % (nb * 8)}
        del buf, evict

    # ---- gather ceilings: whole rows of a table read at random (fuse_probe_gather, the V_j fetch of the
    # Outer template without its arithmetic) from a table that fits one L2, one that fits the memory-side
    # cache (the size of V) and one that fits neither; and from the V-sized table in the order of a panel
    # walk (random inside a 5 MB window that moves through the table).  Stored cells per second of the
    # Outer operator are set against these, not against the HBM peak.
    ceilings = None
    if "outer" in names:
        r = info["outer"]["rank"]
        cnt = 10_000_000
        sink = torch.zeros(1, dtype=torch.float64, device="cuda")

        def gather_rate(rows, idx):
            table = torch.rand(rows, r, dtype=torch.float64, device="cuda")
            best = 0.0
            for blocks in (768, 1024):                     # 3 and 4 resident blocks per CU: the better one counts
                ts = []
                for k in range(7):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    F.probe_gather(table, idx, sink, blocks)
                    b.record()
                    ts.append((a, b))
                torch.cuda.synchronize()
                t = sorted(a.elapsed_time(b) for a, b in ts[2:])[len(ts[2:]) // 2] * 1e-3
                best = max(best, idx.numel() / t)
            return best

        def rnd(rows):
            return torch.randint(0, rows, (cnt,), dtype=torch.int32, device="cuda")

        row_bytes = 8 * r
        sizes = {"l2_resident_2MB": 2_000_000 // row_bytes, "cache_resident_80MB": 80_000_000 // row_bytes,
                 "hbm_resident_2GB": 2_000_000_000 // row_bytes}
        ceilings = {"what": "fuse_probe_gather: %d random rows of %d bytes, 8 lanes per row, 4 rows in flight per group, "
                            "768 or 1024 blocks (the faster); median of 5" % (cnt, row_bytes), "rows_per_s": {}, "GBps": {}}
        for key, rows in sizes.items():
            rate = gather_rate(rows, rnd(rows))
            ceilings["rows_per_s"][key] = float("%.4g" % rate)
            ceilings["GBps"][key] = round(rate * row_bytes / 1e9, 1)
        rows, win = sizes["cache_resident_80MB"], 5_000_000 // row_bytes
        nwin = rows // win
        idx = torch.cat([torch.randint(q * win, (q + 1) * win, (cnt // nwin,), dtype=torch.int32, device="cuda")
                         for q in range(nwin)])
        rate = gather_rate(rows, idx)
        ceilings["rows_per_s"]["80MB_in_5MB_windows"] = float("%.4g" % rate)
        ceilings["GBps"]["80MB_in_5MB_windows"] = round(rate * row_bytes / 1e9, 1)
        del idx

    traffic = profile_traffic()
    traced = profile_kernel_us()
    templates = {}
    for name in names:
        ts = sorted(a.elapsed_time(b) for a, b in ev[name])           # milliseconds
        avg = sum(ts) / len(ts)
        e = {"kernel": kernels[name], "bytes": info[name]["bytes"], "avg_us": round(avg * 1e3, 2),
             "min_us": round(ts[0] * 1e3, 2), "median_us": round(ts[len(ts) // 2] * 1e3, 2),
             "GBps": round(gbps(info[name]["bytes"], avg * 1e-3), 1)}
        e["frac_of_hbm_peak"] = round(e["GBps"] / HBM_PEAK_GBPS, 4)
        tr = traffic.get(kernels[name])
        e["traffic"] = None if tr is None else tr[0] + tr[1]
        if tr is not None:
            e["traffic_GBps"] = round(gbps(tr[0] + tr[1], avg * 1e-3), 1)
        if kernels[name] in traced:
            # the kernel's own duration in the committed kernel trace (the event bracket above also holds the two
            # event records and, for Row and Outer, the small second kernel of a call)
            e["profiled_kernel_us"] = round(traced[kernels[name]], 2)
            if name != "outer":
                e["profiled_kernel_frac_of_hbm_peak"] = round(
                    gbps(info[name]["bytes"], traced[kernels[name]] * 1e-6) / HBM_PEAK_GBPS, 4)
        if info[name]["nnz"]:
            e["nnz_per_s"] = float("%.5g" % (info[name]["nnz"] / (avg * 1e-3)))
        if name == "outer":
            e["bound"] = "l2_gather"
            e["bytes_gather_model"] = info[name]["bytes_gather_model"]
            e["GBps_gather_model"] = round(gbps(info[name]["bytes_gather_model"], avg * 1e-3), 1)
            e["frac_of_l2_gather_ceiling"] = round(e["nnz_per_s"] / ceilings["rows_per_s"]["l2_resident_2MB"], 4)
            e["note"] = ("not HBM-bound: the step's HBM bytes are X, U and V once (GBps, frac_of_hbm_peak); the time goes "
                         "into one V row per stored cell, served by L2 in the column-panel form -- see roofline")
        else:
            e["bound"] = "hbm"
            e["meets_70pct_target"] = bool(e["frac_of_hbm_peak"] >= 0.70)
        if name == "cell" and cell_floor is not None:
            e["plain_read_floor"] = cell_floor
        templates[name] = e
    total_bytes = sum(info[n]["bytes"] for n in names)
    dominant = max(names, key=lambda n: templates[n]["avg_us"])
    d = templates[dominant]
    if dominant == "outer":
        # achieved / peak in bytes of V rows gathered per second (8r per stored cell on both sides)
        row_bytes = 8 * info["outer"]["rank"]
        peak = ceilings["rows_per_s"]["l2_resident_2MB"] * row_bytes / 1e9
        ach = d["nnz_per_s"] * row_bytes / 1e9
        roofline = {"bound": "l2_gather", "kernel": d["kernel"], "template": dominant, "achieved": round(ach, 1),
                    "peak": round(peak, 1), "unit": "GB/s", "frac": round(ach / peak, 4), "traffic": d["traffic"],
                    "note": "Outer is bound by the gather of one V row per stored cell, which its column panels serve from "
                            "L2: achieved = stored cells/s x 8r bytes, peak = the rate fuse_probe_gather reaches on an "
                            "L2-resident table in this run (gather_ceilings); against the HBM peak the same kernel stands at "
                            "frac_of_hbm_peak of its compulsory bytes, and at traffic_GBps of the bytes its L2 misses move"}
    else:
        roofline = {"bound": "hbm", "kernel": d["kernel"], "template": dominant, "achieved": d["GBps"],
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(d["GBps"] / HBM_PEAK_GBPS, 4),
                    "traffic": d["traffic"]}
    hbm_bound = [n for n in names if n != "outer"]
    result = {
        "metric": "effective HBM GB/s of one pass over the five fused templates (bytes each operator must move from "
                  "HBM -- its inputs once -- / step time); per-template fractions of the HBM peak and nnz/s for Outer "
                  "in `templates`",
        "value": round(gbps(total_bytes, elapsed / K), 1), "unit": "GB/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "one launch each of: " + ", ".join(
            {"cell": "Cell sum(X*Y*Z) 1000x1000", "magg": "MAgg [sum(X*Y),sum(X*Z),sum(X^2)] 100000x1000",
             "row_dense": "Row t(X)%*%(w*(X%*%v)) 1e6x100", "row_csr": "Row-CSR t(X)%*%(X%*%v) 1e7x1000 d=0.01",
             "outer": "Outer sum(X*log(U%*%t(V)+1e-15)) 1e5x1e5 d=0.001 r=100"}[n] for n in names),
            "seed": W.BASE_SEED},
        "frac_of_hbm_peak": round(gbps(total_bytes, elapsed / K) / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
        "templates": templates,
        "below_70pct_of_hbm_peak": [n for n in hbm_bound if not templates[n]["meets_70pct_target"]],
        "gather_ceilings": ceilings,
        "plan_cache": {"hits": hits, "misses": misses, "compile_ms": round(compile_ms, 1)},
        "hip_graph_replay": graph,
    }
    if not args.no_cpu_baseline:
        base, refs = _cpu_baseline(names, host, {n: info[n]["bytes"] for n in names})
        result["cpu_baseline"] = base
        # the same run also checks the GPU results against the oracle's
        errs = {}
        for name in names:
            got, ref = outs[name].cpu().numpy(), refs[name]
            if name == "magg":
                errs[name] = float(np.max(np.abs(got - ref) / np.abs(ref)))
            else:
                errs[name] = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        result["max_rel_err_vs_oracle"] = {k: float("%.2e" % v) for k, v in errs.items()}
        assert all(v <= 1e-10 for v in errs.values()), errs
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
