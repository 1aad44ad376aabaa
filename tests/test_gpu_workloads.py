"""GPU parity of the five workloads against the CPU oracle (element by element,
1e-10 relative on fp64 aggregates), at reduced sizes that span several tiles and
a ragged tail and at the full benchmark sizes in the benchmark's launch shape."""
import numpy as np
import pytest

import workloads as W
from oracle import ops, plans, unfused
from gpu_util import to_dev, dev_sides, dev_csr, host, assert_close

pytestmark = pytest.mark.gpu

TOL = 1e-10     # relative tolerance on fp64 aggregates


def _run(w):
    import paper_1801_00829_amd as F
    t = w["template"]
    if t == "cell":
        return host(F.fuse_cell(w["expr"], to_dev(w["X"]), dev_sides(w["sides"]), w["agg"]))
    if t == "magg":
        return host(F.fuse_magg(w["exprs"], to_dev(w["X"]), dev_sides(w["sides"])))
    if t == "row":
        X = w["X"]
        Xd = dev_csr(*X) if isinstance(X, tuple) else to_dev(X)
        return host(F.fuse_row(w["expr"], Xd, dev_sides(w["sides"]), w["agg"]))
    if t == "outer":
        return host(F.fuse_outer(w["expr"], dev_csr(*w["X"]), to_dev(w["U"]), to_dev(w["V"]),
                                 dev_sides(w["sides"]), w["agg"]))
    raise KeyError(t)


def _oracle(name, w):
    if name == "cell":
        return plans.cell_sum_xyz(w["X"], w["sides"][0][1], w["sides"][1][1])
    if name == "magg":
        return plans.magg_xy_xz_xx(w["X"], w["sides"][0][1], w["sides"][1][1])
    if name == "row_dense":
        return plans.row_tx_w_xv(w["X"], w["sides"][0][1], w["sides"][1][1])
    if name == "row_csr":
        return plans.row_csr_tx_xv(ops.make_csr(*w["X"]), w["sides"][0][1])
    return plans.outer_sum_x_log_uv(ops.make_csr(*w["X"]), w["U"], w["V"])


SMALL = [("cell", 0.0377), ("cell", 1.0), ("magg", 0.00211), ("row_dense", 0.00333), ("row_csr", 0.00021),
         ("outer", 0.0123)]


@pytest.mark.parametrize("name,scale", SMALL)
def test_workload_small(name, scale):
    w = W.make_workload(name, scale)
    got, ref = _run(w), _oracle(name, w)
    if name == "magg":          # every aggregate to 1e-10 of its own value
        for j in range(3):
            assert_close(got[j], ref[j], tol=TOL, what="%s[%d]" % (name, j))
    else:
        assert_close(got, ref, tol=TOL, what=name)


@pytest.mark.parametrize("name", ["cell", "magg", "row_dense", "row_csr", "outer"])
def test_workload_full_size(name):
    """The benchmark sizes, launched exactly as the benchmark launches them; the
    oracle computes the full result (a few seconds per workload on the host)."""
    print("full-size parity:", name, flush=True)
    w = W.make_workload(name, 1.0)
    got, ref = _run(w), _oracle(name, w)
    if name == "magg":
        for j in range(3):
            assert_close(got[j], ref[j], tol=TOL, what="%s[%d]" % (name, j))
    else:
        assert_close(got, ref, tol=TOL, what=name)
    # a second launch must give the same bits (deterministic order; ticket reset works)
    if name != "row_csr":
        assert np.array_equal(_run(w), got)
    else:
        assert_close(_run(w), got, tol=1e-13, what="row_csr rerun")


@pytest.mark.parametrize("agg", ["right_mm", "left_mm"])
def test_outer_product_variants_full_size(agg):
    """The two product variants of the Outer template at the benchmark shape (1e5 x 1e5, 1e7 stored cells,
    rank 100) with the weights of the ALS-CG update, (X != 0) * (U t(V)): every output row against the oracle."""
    import paper_1801_00829_amd as F
    print("full-size parity: outer", agg, flush=True)
    w = W.make_workload("outer", 1.0)
    body = [("main",), ("neq0",), ("uvdot",), ("mul",)]
    got = host(F.fuse_outer(body, dev_csr(*w["X"]), to_dev(w["U"]), to_dev(w["V"]), [], agg))
    ref = unfused.outer(body, ops.make_csr(*w["X"]), w["U"], w["V"], [], agg)
    assert_close(got, ref, tol=TOL, what="outer " + agg)
    err = np.abs(got.reshape(ref.shape) - ref) / np.maximum(np.abs(ref), 1e-300)     # all terms are positive here
    assert err.max() <= 1e-12, err.max()


@pytest.mark.parametrize("sides_kind", ["matrix", "vectors"])
def test_cell_variants_at_scale(sides_kind):
    """All four variants of the Cell template (Table 1: no_agg, row_agg, col_agg, full_agg) on 100000 x 1000
    (the size of the paper's Fig. 8 sweep where the inputs no longer fit any cache), every output element
    against the oracle; with a matrix side input (flat form where it applies) and with column- and row-vector
    side inputs (2-D form)."""
    import paper_1801_00829_amd as F
    m, n = 100_000, 1000
    x = W.dense_uniform(m, n, -1.0, 1.0, 991)
    if sides_kind == "matrix":
        sides = [("matrix", W.dense_uniform(m, n, -1.0, 1.0, 992))]
        expr = [("main",), ("side", 0), ("mul",)]
    else:
        sides = [("colvec", W.dense_uniform(m, 1, -1.0, 1.0, 993).reshape(m)),
                 ("rowvec", W.dense_uniform(n, 1, -1.0, 1.0, 994).reshape(n))]
        expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    xd, sd = to_dev(x), dev_sides(sides)
    none_ref = unfused.cell(expr, x, sides, "none").reshape(m, n)
    absv = np.abs(none_ref)
    for agg in ("none", "row", "col", "full"):
        print("cell at scale:", sides_kind, agg, flush=True)
        got = host(F.fuse_cell(expr, xd, sd, agg))
        ref = none_ref if agg == "none" else unfused.cell(expr, x, sides, agg)
        scale = None if agg == "none" else float(absv.sum()) if agg == "full" else \
            float(absv.sum(1).max()) if agg == "row" else float(absv.sum(0).max())
        assert_close(got, np.asarray(ref).reshape(-1), scale=scale, tol=TOL, what="cell %s %s" % (sides_kind, agg))


def test_sparse_cell_with_sparse_sides_at_scale():
    """Fig. 8b / 8d at 100000 x 1000 with X, Y and Z a tenth stored each (1e7 stored cells per matrix, the launch shape
    of the large sweep sizes): sum(X*Y*Z) in all four variants and the two-aggregate MAgg, every output element against
    the oracle's operator-at-a-time plan on the densified side matrices."""
    import paper_1801_00829_amd as F
    m, n = 100_000, 1000
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 981)
    x = ops.make_csr(rp, ci, va, (m, n))
    gpu_sides, ref_sides = [], []
    for seed, rp64 in ((982, False), (983, True)):
        srp, sci, sva = W.csr_bernoulli(m, n, 0.1, seed)
        gpu_sides.append(("sparse", (srp, sci, sva, (m, n), rp64)))
        ref_sides.append(("matrix", ops.csr_to_dense(ops.make_csr(srp, sci, sva, (m, n)))))
    xd, sd = dev_csr(rp, ci, va, (m, n)), dev_sides(gpu_sides)
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    none_ref = unfused.cell_csr(expr, x, ref_sides, "none")
    absv = np.abs(none_ref)
    for agg in ("none", "row", "col", "full"):
        print("sparse cell with sparse sides at scale:", agg, flush=True)
        got = host(F.fuse_cell_csr(expr, xd, sd, agg))
        ref = none_ref if agg == "none" else unfused.cell_csr(expr, x, ref_sides, agg)
        scale = None if agg == "none" else float(absv.sum()) if agg == "full" else \
            float(ops.csr_row_sums(x, absv).max()) if agg == "row" else float(ops.csr_col_sums(x, absv).max())
        assert_close(got, np.asarray(ref).reshape(-1), scale=scale, tol=TOL, what="sparse sides %s" % agg)
    two = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)]]
    got = host(F.fuse_magg_csr(two, xd, sd))
    ref = unfused.magg_csr(two, x, ref_sides)
    for j in range(2):
        a = float(np.abs(unfused.cell_csr(two[j], x, ref_sides, "none")).sum())
        assert_close(got[j], ref[j], scale=a, tol=TOL, what="sparse sides magg[%d]" % j)


def test_long_chain_expression_at_scale():
    """The expression of the paper's instruction-footprint experiment (Sec. 5.3): sum(f(X / rowSums(X))) with f a
    chain of 31 scalar operations, on 30000 x 1000 (the oracle materialises every one of the 33 intermediates);
    the row aggregate feeds the chain, the chain the full aggregate."""
    import paper_1801_00829_amd as F
    m, n = 30_000, 1000
    x = W.dense_uniform(m, n, 0.5, 1.5, 995)
    expr = [("main",), ("main",), ("rowsum",), ("div",)]
    for q in range(31):
        expr += [("const", 1.0 + 1e-3 * (q + 1)), ("mul",)]
    got = host(F.fuse_row(expr, to_dev(x), [], "full"))
    ref = unfused.row_dense(expr, x, [], "full")
    assert_close(got, ref, tol=TOL, what="long chain full")             # all summands positive
    got = host(F.fuse_row(expr, to_dev(x), [], "row"))
    assert_close(got, unfused.row_dense(expr, x, [], "row"), tol=TOL, what="long chain row")


def test_calls_on_two_streams_keep_their_own_workspaces():
    """Every (device, stream) pair has its own block partials and arrival counter: operators that
    overlap on two streams (default priorities) must not disturb each other's aggregates."""
    import torch
    import paper_1801_00829_amd as F
    from oracle import plans
    rng = np.random.default_rng(17)
    xs = [rng.uniform(size=(700, 900)) for _ in range(2)]
    ys = [rng.uniform(size=(700, 900)) for _ in range(2)]
    zs = [rng.uniform(size=(700, 900)) for _ in range(2)]
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    refs = [plans.cell_sum_xyz(xs[i], ys[i], zs[i])[0] for i in range(2)]
    dev = [tuple(torch.from_numpy(a).cuda() for a in (xs[i], ys[i], zs[i])) for i in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[torch.empty(1, dtype=torch.float64, device="cuda") for _ in range(12)] for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(12):
        for i in range(2):
            x, y, z = dev[i]
            F.fuse_cell(expr, x, [("matrix", y), ("matrix", z)], "full", out=outs[i][rep], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        for rep in range(12):
            assert abs(float(outs[i][rep].cpu()[0]) - refs[i]) <= 1e-10 * abs(refs[i]), (i, rep)


def test_full_aggregates_back_to_back_on_changing_inputs():
    """The single-launch finish of a full aggregate reuses one workspace per stream: a block's partial
    sums from the previous call are still there when the next call starts.  Forty calls back to back
    on one stream, every one on different inputs and with as many blocks as the device has compute
    units, must each give their own sum -- a partial that the block with the last ticket read before
    its publisher's store had arrived would be the previous call's (a different number here)."""
    import torch
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(4242)
    m, n, nset = 2100, 1000, 8                                 # 16.8 MB per matrix: one tile run per block and more
    xs = [rng.uniform(-1.0, 1.0, size=(m, n)) * (1.0 + 3.0 * i) for i in range(nset)]
    y, z = rng.uniform(size=(m, n)), rng.uniform(size=(m, n))
    cell = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    magg = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)], [("main",), ("pow2",)]]
    ref_cell = [plans.cell_sum_xyz(x, y, z)[0] for x in xs]
    ref_magg = [plans.magg_xy_xz_xx(x, y, z) for x in xs]
    scale_cell = [float(np.abs(x * y * z).sum()) for x in xs]
    scale_magg = [np.array([np.abs(x * y).sum(), np.abs(x * z).sum(), (x * x).sum()]) for x in xs]
    dx = [to_dev(x) for x in xs]
    sides = dev_sides([("matrix", y), ("matrix", z)])
    reps = 40
    oc = torch.full((reps,), float("nan"), dtype=torch.float64, device="cuda")
    om = torch.full((reps, 3), float("nan"), dtype=torch.float64, device="cuda")
    torch.cuda.synchronize()
    for rep in range(reps):
        i = (rep * 3) % nset                                   # consecutive calls never share an input
        F.fuse_cell(cell, dx[i], sides, "full", out=oc[rep:rep + 1])
        F.fuse_magg(magg, dx[i], sides, out=om[rep])
    gc, gm = host(oc), host(om)
    for rep in range(reps):
        i = (rep * 3) % nset
        assert abs(gc[rep] - ref_cell[i]) <= TOL * scale_cell[i], ("cell", rep, i, gc[rep], ref_cell[i])
        assert (np.abs(gm[rep] - ref_magg[i]) <= TOL * scale_magg[i]).all(), ("magg", rep, i, gm[rep], ref_magg[i])
    # the same for the Outer full aggregate (its own finish after a different main loop)
    w = W.make_workload("outer", 0.03)
    xo, u, v = dev_csr(*w["X"]), to_dev(w["U"]), to_dev(w["V"])
    oo = torch.full((12,), float("nan"), dtype=torch.float64, device="cuda")
    refs = []
    for rep in range(12):
        f = 1.0 + 0.5 * rep
        refs.append(plans.outer_sum_x_log_uv(ops.make_csr(*w["X"]), w["U"] * f, w["V"])[0])
    uf = [to_dev(w["U"] * (1.0 + 0.5 * rep)) for rep in range(12)]
    torch.cuda.synchronize()
    for rep in range(12):
        F.fuse_outer(w["expr"], xo, uf[rep], v, [], "full", out=oo[rep:rep + 1])
    go = host(oo)
    for rep in range(12):
        assert abs(go[rep] - refs[rep]) <= TOL * abs(refs[rep]), ("outer", rep, go[rep], refs[rep])


def test_step_of_five_operators_replays_from_a_hip_graph():
    """After a warm-up on the same stream (plans compiled and loaded, workspace allocated) the calls
    enqueue kernels only, so a whole step can be captured into a HIP graph and replayed without the
    host launch path.  Every replay is checked against the oracle on inputs changed (eagerly) since
    the previous one: arrival counters reset themselves, workspaces are reused, nothing is cached."""
    import torch
    import paper_1801_00829_amd as F
    ws = {n: W.make_workload(n, sc) for n, sc in (("cell", 0.05), ("magg", 0.003), ("row_dense", 0.004),
                                                  ("row_csr", 0.0004), ("outer", 0.02))}
    d = {}
    for n in ("cell", "magg", "row_dense"):
        d[n] = (to_dev(ws[n]["X"]), dev_sides(ws[n]["sides"]))
    d["row_csr"] = (dev_csr(*ws["row_csr"]["X"]), dev_sides(ws["row_csr"]["sides"]))
    d["outer"] = (dev_csr(*ws["outer"]["X"]), to_dev(ws["outer"]["U"]), to_dev(ws["outer"]["V"]))
    outs = {"cell": torch.empty(1, dtype=torch.float64, device="cuda"),
            "magg": torch.empty(3, dtype=torch.float64, device="cuda"),
            "row_dense": torch.empty(ws["row_dense"]["X"].shape[1], dtype=torch.float64, device="cuda"),
            "row_csr": torch.empty(ws["row_csr"]["X"][3][1], dtype=torch.float64, device="cuda"),
            "outer": torch.empty(1, dtype=torch.float64, device="cuda")}

    def step():
        F.fuse_cell(ws["cell"]["expr"], d["cell"][0], d["cell"][1], "full", out=outs["cell"])
        F.fuse_magg(ws["magg"]["exprs"], d["magg"][0], d["magg"][1], out=outs["magg"])
        F.fuse_row(ws["row_dense"]["expr"], d["row_dense"][0], d["row_dense"][1], "col_t", out=outs["row_dense"])
        F.fuse_row(ws["row_csr"]["expr"], d["row_csr"][0], d["row_csr"][1], "col_t", out=outs["row_csr"])
        F.fuse_outer(ws["outer"]["expr"], d["outer"][0], d["outer"][1], d["outer"][2], [], "full", out=outs["outer"])

    def check(tag):
        torch.cuda.synchronize()
        for n in ws:
            got, ref = outs[n].cpu().numpy(), _oracle(n, ws[n])
            if n == "magg":
                for j in range(3):
                    assert_close(got[j], ref[j], tol=TOL, what="%s %s[%d]" % (tag, n, j))
            else:
                assert_close(got, ref, tol=TOL, what="%s %s" % (tag, n))

    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()                                   # warm-up on the capture stream
    s.synchronize()
    check("eager")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        step()
    for rep in range(3):
        # change the inputs in place (eager work between the replays), on the host copies too
        f = 1.0 + 0.25 * (rep + 1)
        for n in ("cell", "magg", "row_dense"):
            d[n][0].mul_(f)
            ws[n]["X"] = ws[n]["X"] * f
        d["row_csr"][0].vals.mul_(f)
        rp, ci, va, shape = ws["row_csr"]["X"]
        ws["row_csr"]["X"] = (rp, ci, va * f, shape)
        d["outer"][1].mul_(f)
        ws["outer"]["U"] = ws["outer"]["U"] * f
        for o in outs.values():
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        print("graph replay", rep, flush=True)
        g.replay()
        check("replay %d" % rep)


def test_cache_clear_between_calls():
    """fuse_cache_clear drops the compiled plans and frees the workspaces (after the caller has synchronised);
    the next calls compile and allocate again and give the same results."""
    import torch
    import paper_1801_00829_amd as F
    w = W.make_workload("row_csr", 0.0005)
    x, s = dev_csr(*w["X"]), dev_sides(w["sides"])
    wc = W.make_workload("cell", 0.05)
    xc, sc = to_dev(wc["X"]), dev_sides(wc["sides"])
    first = (host(F.fuse_row(w["expr"], x, s, "col_t")), host(F.fuse_cell(wc["expr"], xc, sc, "full")))
    for _ in range(2):
        torch.cuda.synchronize()
        F.cache_clear()
        assert F.cache_stats()[:2] == (0, 0)
        again = (host(F.fuse_row(w["expr"], x, s, "col_t")), host(F.fuse_cell(wc["expr"], xc, sc, "full")))
        assert F.cache_stats()[1] == 2                      # both plans were compiled anew
        assert_close(again[0], first[0], tol=1e-13, what="row_csr after clear")
        assert np.array_equal(again[1], first[1])
