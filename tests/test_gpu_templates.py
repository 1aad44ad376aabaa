"""GPU parity of the template skeletons on random expressions, all aggregation
variants, odd shapes and edge cases, against the oracle's operator-at-a-time
evaluation.  Integer / index work (positions of outputs on a CSR pattern,
per-row counts, total nnz) must be bit-exact."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import ops, unfused
from exprgen import random_scalar_expr, random_row_expr
from gpu_util import to_dev, dev_sides, dev_csr, host, assert_close

pytestmark = pytest.mark.gpu

# FUSE_TEST_MORE=k multiplies the number of random-expression cases (seeds) per test; the
# default suite runs k = 1.
MORE = max(1, int(os.environ.get("FUSE_TEST_MORE", "1")))

KINDS = ["matrix", "colvec", "rowvec", "scalar"]


def _sides(rng, m, n, lo=-1.5, hi=1.5):
    return [("matrix", rng.uniform(lo, hi, size=(m, n))), ("colvec", rng.uniform(lo, hi, size=m)),
            ("rowvec", rng.uniform(lo, hi, size=n)), ("scalar", np.array(rng.uniform(lo, hi)))]


def _abs_scale(vals_none, agg, m, n):
    """Aggregate of |summands| in the shape of the result: the natural error scale of a sum."""
    a = np.abs(np.nan_to_num(np.asarray(vals_none, dtype=np.float64), nan=0.0, posinf=0.0, neginf=0.0))
    if agg == "none":
        return None
    a = a.reshape(m, -1)
    if agg == "full":
        return max(a.sum(), 1e-300)
    if agg == "row":
        return max(a.sum(1).max(), 1e-300)
    return max(a.sum(0).max(), 1e-300)


# ------------------------------------------------------------------------- Cell ---

CELL_SHAPES = [(1, 1), (3, 5), (37, 129), (64, 256), (257, 100), (5, 4099), (1000, 3)]


@pytest.mark.parametrize("case", range(14 * MORE))
def test_cell_random_expressions_all_variants(case):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(5000 + case)
    m, n = CELL_SHAPES[case % len(CELL_SHAPES)]
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    x[rng.random((m, n)) < 0.1] = 0.0
    sides = _sides(rng, m, n)
    expr = random_scalar_expr(rng, len(KINDS))
    xd, sd = to_dev(x), dev_sides(sides)
    none_ref = unfused.cell(expr, x, sides, "none")
    for agg in ("none", "full", "row", "col"):
        print("cell case", case, (m, n), agg, expr, flush=True)
        got = host(F.fuse_cell(expr, xd, sd, agg))
        ref = unfused.cell(expr, x, sides, agg)
        assert_close(got, ref, scale=_abs_scale(none_ref, agg, m, n), what="cell %s" % agg)


def test_cell_flat_paths_and_alignment():
    """Contiguous matrix-only bodies take the flat kernel: odd sizes, unaligned bases, no-agg store."""
    import torch
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(7)
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("add",), ("abs",), ("sqrt",)]
    for (m, n) in [(1, 1), (1, 7), (33, 31), (128, 1024), (999, 1001)]:
        x, y, z = rng.uniform(-1, 1, size=(3, m, n))
        ref_none = np.sqrt(np.abs(x * y + z))
        for off in (0, 1):          # off = 1: base pointers 8-byte but not 16-byte aligned
            def dev(a):
                buf = torch.empty(a.size + 1, dtype=torch.float64, device="cuda")
                v = buf[off:off + a.size].view(a.shape)
                v.copy_(torch.from_numpy(a))
                return v
            xd, yd, zd = dev(x), dev(y), dev(z)
            print("cell flat", (m, n), "offset", off, flush=True)
            got = host(F.fuse_cell(expr, xd, [("matrix", yd), ("matrix", zd)], "full"))
            assert_close(got, [ops.sum_full(ref_none)], what="flat full")
            got = host(F.fuse_cell(expr, xd, [("matrix", yd), ("matrix", zd)], "none"))
            assert_close(got, ref_none, tol=1e-12, what="flat none")   # fused multiply-add vs two roundings


def test_cell_strided_views():
    """ld > cols for the main input and a matrix side; a strided column-vector side."""
    import torch
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(8)
    m, n = 50, 70
    xb, yb = rng.uniform(-1, 1, size=(2, m, n + 10))
    cb = rng.uniform(-1, 1, size=(m, 3))
    x, y, c = xb[:, 3:3 + n], yb[:, :n], cb[:, 1]
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("sub",)]
    xd, yd, cd = to_dev(xb)[:, 3:3 + n], to_dev(yb)[:, :n], to_dev(cb)[:, 1:2]
    for agg in ("none", "full", "row", "col"):
        got = host(F.fuse_cell(expr, xd, [("matrix", yd), ("colvec", cd)], agg))
        ref = unfused.cell(expr, x, [("matrix", y), ("colvec", c)], agg)
        assert_close(got, ref, scale=_abs_scale(x * y - c[:, None], agg, m, n), what="strided %s" % agg)


def test_cell_empty_inputs():
    import torch
    import paper_1801_00829_amd as F
    expr = [("main",), ("pow2",)]
    for shape in [(0, 5), (4, 0)]:
        x = torch.empty(shape, dtype=torch.float64, device="cuda")
        assert host(F.fuse_cell(expr, x, [], "full")).tolist() == [0.0]
        assert host(F.fuse_cell(expr, x, [], "row")).tolist() == [0.0] * shape[0]
        assert host(F.fuse_cell(expr, x, [], "col")).tolist() == [0.0] * shape[1]
        assert host(F.fuse_cell(expr, x, [], "none")).size == 0


def test_cell_closed_forms_on_gpu():
    import torch
    import paper_1801_00829_amd as F
    m, n = 777, 333
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    x = torch.full((m, n), 0.5, dtype=torch.float64, device="cuda")
    assert host(F.fuse_cell(expr, x, [("matrix", x), ("matrix", x)], "full"))[0] == m * n * 0.125
    ones = torch.ones((m, n), dtype=torch.float64, device="cuda")
    yi = torch.arange(m, dtype=torch.float64, device="cuda")[:, None].expand(m, n).contiguous()
    zj = torch.arange(n, dtype=torch.float64, device="cuda")[None, :].expand(m, n).contiguous()
    assert host(F.fuse_cell(expr, ones, [("matrix", yi), ("matrix", zj)], "full"))[0] == \
        (m * (m - 1) // 2) * (n * (n - 1) // 2)


# ------------------------------------------------------------------------- MAgg ---

@pytest.mark.parametrize("case", range(6 * MORE))
def test_magg_random_and_equals_separate_cells(case):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(6000 + case)
    m, n = [(1, 1), (19, 23), (300, 129), (64, 1024), (1001, 77), (2, 100001)][case % 6]
    k = int(rng.integers(1, 6))
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    sides = [("matrix", rng.uniform(-1.5, 1.5, size=(m, n))), ("matrix", rng.uniform(-1.5, 1.5, size=(m, n))),
             ("scalar", np.array(0.7))]
    exprs = [random_scalar_expr(rng, 3, depth=3) for _ in range(k)]
    print("magg case", case, (m, n), exprs, flush=True)
    xd, sd = to_dev(x), dev_sides(sides)
    got = host(F.fuse_magg(exprs, xd, sd))
    ref = unfused.magg(exprs, x, sides)
    for j in range(k):
        scale = _abs_scale(unfused.cell(exprs[j], x, sides, "none"), "full", m, n)
        assert_close(got[j], ref[j], scale=scale, what="magg[%d]" % j)
        # a multi-aggregate equals its aggregates computed one by one
        one = host(F.fuse_cell(exprs[j], xd, sd, "full"))
        assert_close(got[j], one[0], scale=scale, tol=1e-13, what="magg vs cell [%d]" % j)


@pytest.mark.parametrize("form", ["flat", "2d", "csr"])
def test_magg_sixteen_aggregates_and_eight_sides(form):
    """The largest multi-aggregate: 16 bodies over 8 side inputs (all matrices: flat form; mixed with
    vectors and scalars: 2-D form; over a sparse main input)."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(6500)
    m, n = 333, 257
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    if form == "flat":
        sides = [("matrix", rng.uniform(-1.5, 1.5, size=(m, n))) for _ in range(8)]
    else:
        sides = [("matrix", rng.uniform(-1.5, 1.5, size=(m, n))), ("colvec", rng.uniform(-1.5, 1.5, size=m)),
                 ("rowvec", rng.uniform(-1.5, 1.5, size=n)), ("scalar", np.array(0.3)),
                 ("matrix", rng.uniform(-1.5, 1.5, size=(m, n))), ("colvec", rng.uniform(-1.5, 1.5, size=m)),
                 ("rowvec", rng.uniform(-1.5, 1.5, size=n)), ("scalar", np.array(-1.1))]
    # body j: X * side_(j % 8) * side_((j + 3) % 8) + X * j   (sparse-safe)
    exprs = [[("main",), ("side", j % 8), ("mul",), ("side", (j + 3) % 8), ("mul",), ("main",), ("const", float(j)), ("mul",),
              ("add",)] for j in range(16)]
    sd = dev_sides(sides)
    if form == "csr":
        rp, ci, va = W.csr_bernoulli(m, n, 0.15, 6501)
        xs = ops.make_csr(rp, ci, va, (m, n))
        got = host(F.fuse_magg_csr(exprs, dev_csr(rp, ci, va, (m, n)), sd))
        ref = unfused.magg_csr(exprs, xs, sides)
        scales = [np.abs(unfused.cell_csr(e, xs, sides, "none")).sum() for e in exprs]
    else:
        got = host(F.fuse_magg(exprs, to_dev(x), sd))
        ref = unfused.magg(exprs, x, sides)
        scales = [np.abs(unfused.cell(e, x, sides, "none")).sum() for e in exprs]
    assert got.shape == (16,)
    for j in range(16):
        assert_close(got[j], ref[j], scale=max(scales[j], 1e-300), what="magg16 %s [%d]" % (form, j))
    with pytest.raises(F.FuseError):
        F.fuse_magg(exprs + [exprs[0]], to_dev(x), sd)            # 17 aggregates


@pytest.mark.parametrize("case", range(6 * MORE))
def test_magg_with_vector_sides_and_strided_inputs(case):
    """MAgg bodies that need the 2-D form of the skeleton: row / column vector sides, views with a
    leading dimension > cols.  Same bar as the flat form, and equal to the aggregates one by one."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(6100 + case)
    m, n = [(1, 1), (19, 23), (300, 129), (64, 1024), (1001, 77), (7, 5000)][case % 6]
    k = int(rng.integers(1, 6))
    pad = [0, 3, 2, 0, 5, 1][case % 6]
    xb, yb = rng.uniform(-1.5, 1.5, size=(m, n + pad)), rng.uniform(-1.5, 1.5, size=(m, n + pad))
    x, y = xb[:, :n], yb[:, :n]
    sides = [("matrix", y), ("colvec", rng.uniform(-1.5, 1.5, size=m)), ("rowvec", rng.uniform(-1.5, 1.5, size=n)),
             ("scalar", np.array(0.7))]
    exprs = [random_scalar_expr(rng, 4, depth=3) for _ in range(k)]
    exprs[0] = [("main",), ("side", 1), ("mul",), ("side", 2), ("mul",)]         # uses both vector sides
    print("magg 2-d case", case, (m, n), "pad", pad, exprs, flush=True)
    xd = to_dev(xb)[:, :n]
    sd = [("matrix", to_dev(yb)[:, :n]), ("colvec", to_dev(sides[1][1])), ("rowvec", to_dev(sides[2][1])),
          ("scalar", 0.7)]
    got = host(F.fuse_magg(exprs, xd, sd))
    assert F.last_kernel().startswith(("fuse_magg2d_", "fuse_cell2d_"))     # 2-D form (a cached 1-body plan keeps its name)
    ref = unfused.magg(exprs, x, sides)
    for j in range(k):
        scale = _abs_scale(unfused.cell(exprs[j], x, sides, "none"), "full", m, n)
        assert_close(got[j], ref[j], scale=scale, what="magg2d[%d]" % j)
        one = host(F.fuse_cell(exprs[j], xd, sd, "full"))
        assert_close(got[j], one[0], scale=scale, tol=1e-13, what="magg2d vs cell [%d]" % j)


def test_cell_bodies_without_a_matrix_operand():
    """A Cell body made of scalars and a column vector only is still a value per CELL: no_agg
    gives m x n values, the aggregates count every cell (2-D form of the skeleton)."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(77)
    for (m, n) in ((1, 1), (5, 3), (70, 130), (300, 64)):
        x = rng.uniform(size=(m, n))
        cv = rng.uniform(1.0, 2.0, size=m)
        sides = [("colvec", cv), ("scalar", np.array(1.5))]
        sd = [("colvec", to_dev(cv)), ("scalar", 1.5)]
        for expr in ([("side", 0)], [("side", 0), ("side", 1), ("mul",), ("const", 0.25), ("add",)]):
            for agg in ("none", "row", "col", "full"):
                print("cell no-matrix", (m, n), expr, agg, flush=True)
                got = host(F.fuse_cell(expr, to_dev(x), sd, agg))
                ref = unfused.cell(expr, x, sides, agg)
                assert got.size == ref.size
                assert_close(got.reshape(ref.shape), ref, scale=_abs_scale(unfused.cell(expr, x, sides, "none"), agg, m, n),
                             what="cell no-matrix %s" % agg)


# -------------------------------------------------------------------- Row dense ---

ROW_SHAPES = [(1, 1), (5, 3), (70, 10), (33, 100), (129, 101), (40, 784), (17, 1000), (9, 2048), (300, 64)]


@pytest.mark.parametrize("case", range(18 * MORE))
def test_row_dense_random_expressions(case):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(7000 + case)
    m, n = ROW_SHAPES[case % len(ROW_SHAPES)]
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    sides = _sides(rng, m, n)
    want = "V" if case % 3 else "S"
    expr = random_row_expr(rng, KINDS, depth=3, want=want)
    xd, sd = to_dev(x), dev_sides(sides)
    none_ref = unfused.row_dense(expr, x, sides, "none")
    for agg in (("none", "row", "col", "col_t", "full") if want == "V" else ("none", "full")):
        print("row dense case", case, (m, n), agg, expr, flush=True)
        got = host(F.fuse_row(expr, xd, sd, agg))
        ref = unfused.row_dense(expr, x, sides, agg)
        scale = _abs_scale(none_ref, agg, m, n if want == "V" else 1)
        assert_close(got, ref, scale=scale, tol=1e-10, what="row dense %s" % agg)


@pytest.mark.parametrize("shape", [(7, 2050), (33, 3000), (12, 4097), (5, 9000), (3, 20000), (2, 32768)])
def test_row_dense_wide_rows_with_reductions(shape):
    """Rows wider than one wave's registers (2048 columns): several waves own a row and
    exchange their partial row aggregates through shared memory."""
    import paper_1801_00829_amd as F
    m, n = shape
    rng = np.random.default_rng(7100 + n)
    x = rng.normal(size=(m, n))
    sides = _sides(rng, m, n)
    xd, sd = to_dev(x), dev_sides(sides)
    exprs = {"V": [("main",), ("side", 2), ("dot",), ("main",), ("mul",), ("main",), ("rowsum",), ("side", 1), ("mul",), ("add",)],
             "S": [("main",), ("side", 0), ("mul",), ("rowsum",), ("main",), ("main",), ("rowsum",), ("sub",), ("pow2",), ("rowsum",), ("add",)]}
    for want, expr in exprs.items():
        none_ref = unfused.row_dense(expr, x, sides, "none")
        for agg in (("none", "row", "col_t", "full") if want == "V" else ("none", "full")):
            print("row wide", shape, want, agg, flush=True)
            got = host(F.fuse_row(expr, xd, sd, agg))
            ref = unfused.row_dense(expr, x, sides, agg)
            scale = _abs_scale(none_ref, agg.replace("col_t", "col"), m, n) if want == "V" else \
                (None if agg == "none" else max(np.abs(none_ref).sum(), 1e-300))
            assert_close(got.reshape(ref.shape), ref, scale=scale, tol=1e-10, what="row wide %s %s" % (want, agg))
    src = F.last_source()
    assert int(src[src.index("#define FUSE_WPR ") + 17:].split()[0]) > 1          # the generator's own definition


def test_row_dense_closed_forms_and_odd_layouts():
    import torch
    import paper_1801_00829_amd as F
    expr = [("main",), ("side", 0), ("dot",), ("side", 1), ("mul",), ("main",), ("mul",)]
    for (m, n) in [(64, 10), (1000, 100), (777, 101), (50, 1000)]:
        x = torch.ones((m, n), dtype=torch.float64, device="cuda")
        v = torch.ones(n, dtype=torch.float64, device="cuda")
        w = torch.ones(m, dtype=torch.float64, device="cuda")
        assert host(F.fuse_row(expr, x, [("rowvec", v), ("colvec", w)], "col_t")).tolist() == [float(m * n)] * n
    # ld > cols and an unaligned row-vector
    rng = np.random.default_rng(9)
    m, n = 333, 100
    xb = rng.normal(size=(m, n + 6))
    vb, w = rng.normal(size=n + 1), rng.uniform(size=m)
    x, v = xb[:, 2:2 + n], vb[1:]
    got = host(F.fuse_row(expr, to_dev(xb)[:, 2:2 + n], [("rowvec", to_dev(vb)[1:]), ("colvec", to_dev(w))], "col_t"))
    from oracle import plans
    assert_close(got, plans.row_tx_w_xv(x, v, w), what="row strided")


NARROW_SHAPES = [(600011, 2), (300007, 8), (150001, 29), (100003, 30), (70001, 50), (66003, 63), (40001, 101),
                 (1, 8), (5, 29), (129, 7), (64, 1), (4097, 3)]


@pytest.mark.parametrize("form", ["staged", "direct"])
@pytest.mark.parametrize("shape", NARROW_SHAPES)
def test_row_dense_narrow_rows(shape, form, monkeypatch):
    """Narrow contiguous rows and odd row lengths: the waves fetch the contiguous span of their rows with
    16-byte loads and hand it out through shared memory (the row counts span several passes of every wave
    and a ragged last span); FUSE_ROW_LDSX=0 keeps the direct loads covered.  Matrix and column-vector
    sides keep their direct loads and must still line up with the rows."""
    import paper_1801_00829_amd as F
    monkeypatch.setenv("FUSE_ROW_LDSX", "1" if form == "staged" else "0")
    F.cache_clear()              # last_source() is the text of the last compilation: compile here
    m, n = shape
    rng = np.random.default_rng(7300 + 13 * n + m % 97)
    x = rng.uniform(-1.5, 1.5, size=(m, n))
    sides = _sides(rng, m, n)
    xd, sd = to_dev(x), dev_sides(sides)
    expr = [("main",), ("side", 2), ("dot",), ("side", 1), ("mul",), ("main",), ("mul",), ("side", 0), ("add",)]
    none_ref = unfused.row_dense(expr, x, sides, "none")
    for agg in ("none", "row", "col_t", "full"):
        print("row narrow", shape, form, agg, flush=True)
        got = host(F.fuse_row(expr, xd, sd, agg))
        ref = unfused.row_dense(expr, x, sides, agg)
        assert_close(got.reshape(ref.shape), ref, scale=_abs_scale(none_ref, agg.replace("col_t", "col"), m, n),
                     tol=1e-10, what="row narrow %s" % agg)
        assert ("#define FUSE_LDSX 1" in F.last_source()) == (form == "staged")
    # per-row scalar results
    expr_s = [("main",), ("side", 2), ("dot",), ("side", 1), ("add",)]
    got = host(F.fuse_row(expr_s, xd, sd, "none"))
    assert_close(got.reshape(-1), unfused.row_dense(expr_s, x, sides, "none").reshape(-1), tol=1e-10, what="row narrow scalar")


def test_row_dense_narrow_rows_with_a_row_stride_are_loaded_directly():
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(7400)
    m, n = 5000, 8
    xb = rng.normal(size=(m, n + 4))
    v = rng.normal(size=n)
    expr = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    F.cache_clear()
    got = host(F.fuse_row(expr, to_dev(xb)[:, 2:2 + n], [("rowvec", to_dev(v))], "col_t"))
    assert "#define FUSE_LDSX 0" in F.last_source()
    assert_close(got, unfused.row_dense(expr, xb[:, 2:2 + n], [("rowvec", v)], "col_t").reshape(-1),
                 scale=np.abs((xb[:, 2:2 + n] @ v)[:, None] * xb[:, 2:2 + n]).sum(0).max(), what="row narrow strided")


def test_row_dense_empty_and_limits():
    import torch
    import paper_1801_00829_amd as F
    expr = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    x = torch.empty((0, 8), dtype=torch.float64, device="cuda")
    v = torch.ones(8, dtype=torch.float64, device="cuda")
    assert host(F.fuse_row(expr, x, [("rowvec", v)], "col_t")).tolist() == [0.0] * 8
    big = torch.ones((2, 4098), dtype=torch.float64, device="cuda")          # several waves per row
    got = host(F.fuse_row(expr, big, [("rowvec", torch.ones(4098, dtype=torch.float64, device="cuda"))], "col_t"))
    assert got.tolist() == [2.0 * 4098] * 4098
    huge = torch.ones((2, 40000), dtype=torch.float64, device="cuda")
    with pytest.raises(F.FuseError) as e:
        F.fuse_row(expr, huge, [("rowvec", torch.ones(40000, dtype=torch.float64, device="cuda"))], "col_t")
    assert e.value.code == -7


# ---------------------------------------------------------------------- Row CSR ---

def _csr_cases():
    yield "bernoulli", W.csr_bernoulli(500, 300, 0.03, 101), (500, 300)
    yield "fixed10", W.csr_fixed_per_row(257, 1000, 10, 102), (257, 1000)
    yield "skewed", W.csr_skewed(400, 900, 0.01, 4, 0.7, 103), (400, 900)
    yield "dense", W.csr_bernoulli(40, 70, 1.0, 104), (40, 70)
    yield "one_row", W.csr_bernoulli(1, 5000, 0.3, 105), (1, 5000)
    yield "one_col", W.csr_bernoulli(3000, 1, 0.5, 106), (3000, 1)
    rp = np.zeros(301, dtype=np.int64)
    yield "all_empty", (rp, np.zeros(0, np.int32), np.zeros(0)), (300, 50)
    rp, ci, va = W.csr_bernoulli(200, 64, 0.2, 107)
    keep = np.repeat(np.arange(200) % 3 != 0, np.diff(rp))       # empty every third row
    counts = np.where(np.arange(200) % 3 != 0, np.diff(rp), 0)
    rp2 = np.zeros(201, np.int64)
    np.cumsum(counts, out=rp2[1:])
    yield "many_empty_rows", (rp2, ci[keep], va[keep]), (200, 64)


@pytest.fixture(params=["groups", "groups_dealt", "stream"])
def csr_mapping(request, monkeypatch):
    """Both CSR Row skeletons: a lane group per row, or waves streaming runs of whole rows
    (by default chosen from the mean row length).  The lane-group form gives every block one
    contiguous row range balanced by rows + stored cells ("groups"; the default for small matrices) or
    deals the rows to the blocks round-robin in pieces of one or three block steps ("groups_dealt"; pieces
    of one step are the default for large matrices)."""
    monkeypatch.setenv("FUSE_CSR_STREAM", "1" if request.param == "stream" else "0")
    if request.param == "groups":
        monkeypatch.setenv("FUSE_CSR_ILV", "0")
    elif request.param == "groups_dealt":
        monkeypatch.setenv("FUSE_CSR_ILV", "1" if request.node.name.count("1") % 2 else "3")
    return request.param


@pytest.mark.parametrize("rowptr64", [False, True])
def test_row_csr_workload_expression_on_all_patterns(rowptr64, csr_mapping):
    import paper_1801_00829_amd as F
    from oracle import plans
    expr = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    for name, (rp, ci, va), shape in _csr_cases():
        print("row csr pattern", name, shape, "rowptr64" if rowptr64 else "rowptr32", flush=True)
        v = np.random.default_rng(3).normal(size=shape[1])
        got = host(F.fuse_row(expr, dev_csr(rp, ci, va, shape, rowptr64), [("rowvec", to_dev(v))], "col_t"))
        x = ops.make_csr(rp, ci, va, shape)
        ref = plans.row_csr_tx_xv(x, v)
        q = ops.csr_matvec(x, np.abs(v))
        scale = max(np.abs(ops.csr_t_matvec(x, q)).max(), 1e-300) if va.size else 1.0
        assert_close(got, ref, scale=scale, what="row csr " + name)


def test_row_csr_index_handling_is_bit_exact(csr_mapping):
    """Counts and positions: with X = 1 on its pattern, row / column / full sums of
    the body `X` are integer counts; the no-agg output must sit at the exact positions."""
    import paper_1801_00829_amd as F
    for name, (rp, ci, va), shape in _csr_cases():
        print("row csr exact", name, flush=True)
        m, n = shape
        xd = dev_csr(rp, ci, np.ones_like(va), shape)
        body = [("main",)]
        assert np.array_equal(host(F.fuse_row(body, xd, [], "row")), np.diff(rp).astype(np.float64))
        assert np.array_equal(host(F.fuse_row(body, xd, [], "col")), np.bincount(ci, minlength=n).astype(np.float64))
        assert host(F.fuse_row(body, xd, [], "full"))[0] == float(rp[-1])
        # positions: out[p] = X_p * colvec[row(p)] * rowvec[col(p)] with integer-valued sides
        rows = np.repeat(np.arange(m), np.diff(rp))
        cv, rv = np.arange(m, dtype=np.float64) + 1, np.arange(n, dtype=np.float64) + 1
        e2 = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
        got = host(F.fuse_row(e2, xd, [("colvec", to_dev(cv)), ("rowvec", to_dev(rv))], "none"))
        assert np.array_equal(got, cv[rows] * rv[ci])


@pytest.mark.parametrize("rowptr64", [False, True])
def test_check_csr_accepts_every_pattern_and_names_each_violation(rowptr64):
    """The structure check passes all generated patterns and reports each kind of planted
    damage with the row that shows it (the check itself never reads outside the arrays)."""
    import paper_1801_00829_amd as F
    for name, (rp, ci, va), shape in _csr_cases():
        print("check csr ok", name, flush=True)
        F.check_csr(dev_csr(rp, ci, va, shape, rowptr64))
    rp, ci, va = W.csr_fixed_per_row(120, 90, 6, 108)
    shape, nnz = (120, 90), int(rp[-1])

    def expect(what, rp_, ci_, text, nnz_=None):
        print("check csr bad:", what, flush=True)
        x = dev_csr(rp_, ci_, va, shape, rowptr64)
        if nnz_ is not None:          # arrays keep their length; only the declared count differs
            x = F.Csr(x.rowptr, x.colidx[:nnz_], x.vals[:nnz_], shape)
        with pytest.raises(F.FuseError) as err:
            F.check_csr(x)
        assert err.value.code == -2          # FUSE_ESHAPE
        assert text in str(err.value), (what, str(err.value))

    r = 37
    bad = rp.copy(); bad[0] = 1
    expect("first offset", bad, ci, "rowptr[0] is not 0")
    bad = rp.copy(); bad[r + 1] = bad[r] - 1
    expect("decreasing offsets", bad, ci, "at row %d" % r)
    bad = rp.copy(); bad[r + 1] = nnz + 5
    expect("offset past the arrays", bad, ci, "at row %d" % r)
    bad = rp.copy(); bad[-1] = nnz - 2
    expect("last offset below nnz", bad, ci, "rowptr[rows] differs from nnz")
    expect("declared nnz below the last offset", rp, ci, "leave [0, nnz] at row %d" % (shape[0] - 1), nnz_=nnz - 3)
    p = int(rp[r]) + 2
    bad = ci.copy(); bad[p] = shape[1]
    expect("column == cols", rp, bad, "outside [0, cols) in row %d" % r)
    bad = ci.copy(); bad[int(rp[r])] = -1
    expect("negative column", rp, bad, "outside [0, cols) in row %d" % r)
    bad = ci.copy(); bad[p], bad[p + 1] = bad[p + 1], bad[p]
    expect("unsorted columns", rp, bad, "not strictly ascending in row %d" % r)
    bad = ci.copy(); bad[p + 1] = bad[p]
    expect("duplicate column", rp, bad, "not strictly ascending in row %d" % r)
    # the last column of one row may exceed the first of the next: rows are independent
    bad = ci.copy(); bad[int(rp[r + 1]) - 1] = shape[1] - 1; bad[int(rp[r + 1])] = 0
    F.check_csr(dev_csr(rp, bad, va, shape, rowptr64))


@pytest.mark.parametrize("case", range(12 * MORE))
def test_row_csr_random_sparse_safe_expressions(case, csr_mapping):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(8000 + case)
    m, n = [(1, 1), (37, 19), (300, 257), (64, 1000), (513, 40), (100, 3000)][case % 6]
    rp, ci, va = W.csr_bernoulli(m, n, [0.5, 0.2, 0.04, 0.01, 0.3, 0.005][case % 6], 8000 + case)
    x = ops.make_csr(rp, ci, va, (m, n))
    sides = _sides(rng, m, n)
    want = "V" if case % 3 else "S"
    expr = random_row_expr(rng, KINDS, depth=3, want=want, sparse_safe=True)
    xd, sd = dev_csr(rp, ci, va, (m, n)), dev_sides(sides)
    none_ref = unfused.row_csr(expr, x, sides, "none")
    for agg in (("none", "row", "col", "col_t", "full") if want == "V" else ("none", "full")):
        print("row csr case", case, (m, n), agg, expr, flush=True)
        got = host(F.fuse_row(expr, xd, sd, agg))
        ref = unfused.row_csr(expr, x, sides, agg)
        if want == "V" and agg != "none":
            a = np.abs(np.nan_to_num(none_ref, nan=0.0, posinf=0.0, neginf=0.0))
            scale = {"full": a.sum(), "row": ops.csr_row_sums(x, a).max(initial=0.0),
                     "col": ops.csr_col_sums(x, a).max(initial=0.0)}[agg.replace("col_t", "col")]
        elif want == "S" and agg == "full":
            scale = np.abs(np.nan_to_num(none_ref, nan=0.0, posinf=0.0, neginf=0.0)).sum()
        else:
            scale = None
        assert_close(got, ref, scale=None if scale is None else max(scale, 1e-300), tol=1e-10,
                     what="row csr %s" % agg)


def test_row_csr_column_sums_of_wide_matrices(csr_mapping):
    """More columns than a per-block shared-memory vector holds: column sums go through fp64
    atomics on the output.  Counts are exact, t(X)(Xv) within the usual bar."""
    import paper_1801_00829_amd as F
    from oracle import plans
    for (m, n, d) in ((3000, 20000, 0.0005), (500, 100001, 0.0002), (40, 19000, 0.2)):
        rp, ci, va = W.csr_bernoulli(m, n, d, 4242)
        print("wide csr", (m, n), "nnz", int(rp[-1]), csr_mapping, flush=True)
        xd = dev_csr(rp, ci, np.ones_like(va), (m, n))
        assert np.array_equal(host(F.fuse_row([("main",)], xd, [], "col")), np.bincount(ci, minlength=n).astype(np.float64))
        assert "#define FUSE_COLS_GLOBAL 1" in F.last_source()
        v = np.random.default_rng(5).normal(size=n)
        expr = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
        got = host(F.fuse_row(expr, dev_csr(rp, ci, va, (m, n)), [("rowvec", to_dev(v))], "col_t"))
        x = ops.make_csr(rp, ci, va, (m, n))
        ref = plans.row_csr_tx_xv(x, v)
        scale = max(np.abs(ops.csr_t_matvec(x, ops.csr_matvec(x, np.abs(v)))).max(), 1e-300)
        assert_close(got, ref, scale=scale, what="wide csr t(X)(Xv)")


def test_row_csr_rejects_programs_that_are_not_sparse_safe():
    import paper_1801_00829_amd as F
    rp, ci, va = W.csr_bernoulli(10, 10, 0.3, 1)
    xd = dev_csr(rp, ci, va, (10, 10))
    with pytest.raises(F.FuseError) as e:
        F.fuse_row([("main",), ("const", 1.0), ("add",)], xd, [], "col")
    assert e.value.code == -3


# ------------------------------------------------------------------------ Outer ---

@pytest.fixture(params=["rows", "panels", "flat", "stationary"])
def outer_mapping(request, monkeypatch):
    """The mappings of the no_agg / full_agg Outer skeleton: a wave per row, or column panels of V
    (forced here with tiny panels; by default only chosen when V overflows an L2) with a lane group
    per row ("panels"), with the cells of a chunk of rows dealt to the groups as one list ("flat"), or
    with the rows of U stationary in LDS while the waves walk all panels ("stationary", the default
    when the rank allows it)."""
    if request.param == "rows":
        monkeypatch.setenv("FUSE_OUTER_PANELS", "0")
    else:
        monkeypatch.setenv("FUSE_OUTER_PANELS", "2")
        monkeypatch.setenv("FUSE_OUTER_PANEL_KB", "1")
        monkeypatch.setenv("FUSE_OUTER_STATIONARY", "1" if request.param == "stationary" else "0")
        monkeypatch.setenv("FUSE_OUTER_FLAT", "1" if request.param == "flat" else "0")
    return request.param


OUTER_FORM = {"rows": 0, "panels": 1, "flat": 2, "stationary": 3}


@pytest.mark.parametrize("case", range(12 * MORE))
def test_outer_random_expressions(case, outer_mapping):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(9000 + case)
    m, n, r = [(1, 1, 1), (30, 20, 7), (200, 300, 100), (64, 64, 20), (500, 100, 33), (40, 2000, 128)][case % 6]
    dens = [1.0, 0.3, 0.02, 0.1, 0.05, 0.01][case % 6]
    rp, ci, va = W.csr_bernoulli(m, n, dens, 9000 + case)
    x = ops.make_csr(rp, ci, va, (m, n))
    u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
    sides = _sides(rng, m, n)
    expr = random_scalar_expr(rng, len(KINDS), extra_leaf="uvdot") if case >= 2 else \
        [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]
    xd, ud, vd, sd = dev_csr(rp, ci, va, (m, n)), to_dev(u), to_dev(v), dev_sides(sides)
    none_ref = unfused.outer(expr, x, u, v, sides, "none")
    for agg in ("none", "full"):
        print("outer case", case, (m, n, r), agg, expr, flush=True)
        got = host(F.fuse_outer(expr, xd, ud, vd, sd, agg))
        ref = unfused.outer(expr, x, u, v, sides, agg)
        scale = None if agg == "none" else max(np.abs(np.nan_to_num(none_ref, nan=0, posinf=0, neginf=0)).sum(), 1e-300)
        assert_close(got, ref, scale=scale, tol=1e-10, what="outer %s" % agg)


def test_outer_closed_forms_patterns_and_index_exactness(outer_mapping):
    import math
    import paper_1801_00829_amd as F
    body = [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]
    for name, (rp, ci, va), shape in _csr_cases():
        m, n = shape
        for r in (100, 7):
            print("outer pattern", name, shape, "rank", r, flush=True)
            xd = dev_csr(rp, ci, np.ones_like(va), shape)
            u, v = np.ones((m, r)), np.ones((n, r))
            got = host(F.fuse_outer(body, xd, to_dev(u), to_dev(v), [], "full"))[0]
            assert abs(got - va.size * math.log(r + 1e-15)) <= 1e-12 * max(1.0, va.size * math.log(r + 1e-15))
            # exact index handling: uvdot alone with U_i = (i+1) e_0, V_j = (j+1) e_0 gives (i+1)(j+1) at p
            u2, v2 = np.zeros((m, r)), np.zeros((n, r))
            u2[:, 0], v2[:, 0] = np.arange(m) + 1, np.arange(n) + 1
            got = host(F.fuse_outer([("uvdot",)], xd, to_dev(u2), to_dev(v2), [], "none"))
            rows = np.repeat(np.arange(m), np.diff(rp))
            assert np.array_equal(got, (rows + 1.0) * (ci + 1.0))
            # number of processed stored cells == rowptr[m]
            host(xd.vals)                         # (synchronises) the source of the next call is inspected:
            F.cache_clear()                       # make sure that it is compiled now, not found in the cache
            assert host(F.fuse_outer([("main",), ("neq0",)], xd, to_dev(u2), to_dev(v2), [], "full"))[0] == float(rp[-1])
            if n > 1 and va.size:
                form = OUTER_FORM[outer_mapping]
                if form == 3 and r > 2000:                     # too few rows of U fit into LDS: the flat form
                    form = 2
                assert "#define FUSE_PANELS %d\n" % form in F.last_source(), outer_mapping
    # zero rows of U: every stored cell of those rows contributes x * log(1e-15)
    rp, ci, va = W.csr_bernoulli(60, 50, 0.2, 11)
    u = np.ones((60, 100))
    u[::2] = 0.0
    x = ops.make_csr(rp, ci, va, (60, 50))
    from oracle import plans
    got = host(F.fuse_outer(body, dev_csr(rp, ci, va, (60, 50)), to_dev(u), to_dev(np.ones((50, 100))), [], "full"))
    assert_close(got, plans.outer_sum_x_log_uv(x, u, np.ones((50, 100))), what="outer zero rows")


@pytest.mark.parametrize("r", [1, 2, 513, 1000, 1024])
def test_outer_extreme_ranks(r, outer_mapping):
    """The smallest and the largest ranks the Outer template takes (1 <= r <= 1024), all variants."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(1300 + r)
    m, n = 70, 90
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 1300 + r)
    x = ops.make_csr(rp, ci, va, (m, n))
    u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
    body = [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]
    xd, ud, vd = dev_csr(rp, ci, va, (m, n)), to_dev(u), to_dev(v)
    for agg in ("full", "none", "right_mm", "left_mm"):
        got = host(F.fuse_outer(body, xd, ud, vd, [], agg))
        ref = unfused.outer(body, x, u, v, [], agg)
        assert_close(got, ref, tol=1e-10, what="outer rank %d %s" % (r, agg))
    with pytest.raises(F.FuseError):
        F.fuse_outer(body, xd, to_dev(rng.uniform(size=(m, 1025))), to_dev(rng.uniform(size=(n, 1025))), [], "full")


def test_outer_rowptr64_and_strided_factors(outer_mapping):
    import paper_1801_00829_amd as F
    from oracle import plans
    rng = np.random.default_rng(12)
    m, n, r = 150, 130, 100
    rp, ci, va = W.csr_bernoulli(m, n, 0.05, 13)
    ub, vb = rng.uniform(size=(m, r + 4)), rng.uniform(size=(n, r + 3))
    x = ops.make_csr(rp, ci, va, (m, n))
    ref = plans.outer_sum_x_log_uv(x, ub[:, :r], vb[:, :r])
    body = [("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)]
    for rp64 in (False, True):
        got = host(F.fuse_outer(body, dev_csr(rp, ci, va, (m, n), rp64), to_dev(ub)[:, :r], to_dev(vb)[:, :r], [], "full"))
        assert_close(got, ref, what="outer strided rp64=%s" % rp64)


# ------------------------------------------------- Outer right_mm / left_mm ---

ALS_W = [("main",), ("neq0",), ("uvdot",), ("mul",)]        # (X != 0) * (U_i . V_j): the ALS-CG update, Sec. 2.2


@pytest.fixture(params=["transposed", "transposed_plain_sort", "atomics"])
def left_mm_form(request, monkeypatch):
    """The forms of left_mm: over the transposed pattern of X (built per call by a two-level counting sort,
    the default; or by the plain one that very wide matrices take), or a scatter with fp64 atomics."""
    monkeypatch.setenv("FUSE_OUTER_LEFT_TRANSPOSE", "0" if request.param == "atomics" else "1")
    monkeypatch.setenv("FUSE_TRANSPOSE_PLAIN", "1" if request.param == "transposed_plain_sort" else "0")
    return request.param


def _outer_mm_on_all_patterns(agg, rowptr64, left_mm_form):
    import paper_1801_00829_amd as F
    for name, (rp, ci, va), shape in _csr_cases():
        m, n = shape
        for r in (100, 7, 20):
            print("outer", agg, name, shape, "rank", r, flush=True)
            rng = np.random.default_rng(31)
            u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
            x = ops.make_csr(rp, ci, va, shape)
            got = host(F.fuse_outer(ALS_W, dev_csr(rp, ci, va, shape, rowptr64), to_dev(u), to_dev(v), [], agg))
            if agg == "left_mm" and va.size:
                assert ("#define FUSE_TRANSPOSED 1" in F.last_source()) == left_mm_form.startswith("transposed")
            ref = unfused.outer(ALS_W, x, u, v, [], agg)
            assert_close(got, ref, scale=max(np.abs(ref).max(), 1e-300) if ref.size else 1.0, what="outer %s %s" % (agg, name))
            # rows / columns without stored cells must be exactly zero
            empty = (np.diff(rp) == 0) if agg == "right_mm" else (np.bincount(ci, minlength=n) == 0)
            assert not got.reshape(-1, r)[empty].any()


def test_outer_right_mm_on_all_patterns():
    _outer_mm_on_all_patterns("right_mm", False, "")


@pytest.mark.parametrize("rowptr64", [False, True])
def test_outer_left_mm_on_all_patterns(rowptr64, left_mm_form):
    _outer_mm_on_all_patterns("left_mm", rowptr64, left_mm_form)


@pytest.mark.parametrize("rowptr64", [False, True])
def test_outer_left_mm_over_a_prepared_pattern(rowptr64):
    """fuse_outer_left: the column-sorted pattern of X is prepared once and reused while U and V -- and, after a
    fuse_outer_left_values call, the values of X -- change from call to call (the ALS-CG loop of Sec. 2.2 evaluates its update on the same X in every iteration);
    every call against the oracle and against fuse_outer LEFT_MM, which sorts per call."""
    import torch
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(4100 + rowptr64)
    body = [("main",), ("uvdot",), ("mul",), ("side", 0), ("add",)]              # looks at the value and at a side input at (i, j)
    for name, (rp, ci, va), shape in _csr_cases():
        m, n = shape
        r = 20
        xd = dev_csr(rp, ci, va, shape, rowptr64)
        pattern = F.outer_left_prepare(xd)
        side = rng.uniform(size=(m, n))
        sd = dev_sides([("matrix", side)])
        for it in range(3):
            print("prepared left_mm", name, shape, "call", it, flush=True)
            vals = va * (1.0 + it) + 0.25 * it
            u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
            xd.vals.copy_(torch.from_numpy(vals))                                    # same structure, new values
            if it:
                F.outer_left_values(xd, pattern)
            ud, vd = to_dev(u), to_dev(v)
            got = host(F.fuse_outer_left(body, xd, pattern, ud, vd, sd))
            x = ops.make_csr(rp, ci, vals, shape)
            ref = unfused.outer(body, x, u, v, [("matrix", side)], "left_mm")
            w_abs = np.abs(unfused.outer(body, x, u, v, [("matrix", side)], "none"))
            absref = ops.csr_t_matmul_dense(x, w_abs, np.abs(u))
            assert_close(got, ref, scale=max(absref.max(initial=0.0), 1e-300), tol=1e-10, what="prepared left_mm " + name)
            per_call = host(F.fuse_outer(body, xd, ud, vd, sd, "left_mm"))
            assert_close(got, per_call, scale=max(absref.max(initial=0.0), 1e-300), tol=1e-12, what="prepared vs per call " + name)
            assert np.array_equal(got, host(F.fuse_outer_left(body, xd, pattern, ud, vd, sd)))      # one pattern: one order of sums


@pytest.mark.parametrize("case", range(8 * MORE))
def test_outer_mm_random_expressions(case, left_mm_form):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(9500 + case)
    m, n, r = [(1, 1, 1), (30, 20, 7), (200, 300, 100), (64, 64, 20)][case % 4]
    dens = [1.0, 0.3, 0.02, 0.1][case % 4]
    rp, ci, va = W.csr_bernoulli(m, n, dens, 9500 + case)
    x = ops.make_csr(rp, ci, va, (m, n))
    u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
    sides = _sides(rng, m, n)
    expr = random_scalar_expr(rng, len(KINDS), extra_leaf="uvdot")
    xd, ud, vd, sd = dev_csr(rp, ci, va, (m, n)), to_dev(u), to_dev(v), dev_sides(sides)
    w_abs = np.abs(np.nan_to_num(unfused.outer(expr, x, u, v, sides, "none"), nan=0, posinf=0, neginf=0))
    for agg in ("right_mm", "left_mm"):
        print("outer mm case", case, (m, n, r), agg, expr, flush=True)
        got = host(F.fuse_outer(expr, xd, ud, vd, sd, agg))
        ref = unfused.outer(expr, x, u, v, sides, agg)
        scale = unfused.outer([("side", 0)], x, u, v, [("matrix", np.zeros((m, n)))], agg)   # shape only
        absref = ops.csr_matmul_dense(x, w_abs, np.abs(v)) if agg == "right_mm" else ops.csr_t_matmul_dense(x, w_abs, np.abs(u))
        assert_close(got, ref, scale=max(absref.max(initial=0.0), 1e-300), tol=1e-10, what="outer mm %s" % agg)


def test_outer_right_mm_unaligned_output_and_odd_rank():
    import torch
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(41)
    m, n = 90, 70
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 42)
    x = ops.make_csr(rp, ci, va, (m, n))
    for r in (6, 5):
        u, v = rng.uniform(size=(m, r)), rng.uniform(size=(n, r))
        buf = torch.zeros(m * r + 1, dtype=torch.float64, device="cuda")
        out = buf[1:]                                   # 8-byte aligned only
        F.fuse_outer(ALS_W, dev_csr(rp, ci, va, (m, n)), to_dev(u), to_dev(v), [], "right_mm", out=out)
        assert_close(host(out), unfused.outer(ALS_W, x, u, v, [], "right_mm"), what="right_mm unaligned r=%d" % r)


def test_als_cg_update_as_two_fused_operators():
    """O = ((X != 0) * (U t(V))) V + 1e-6 * U * r  (Sec. 2.2, first example expression): the Outer
    right_mm operator followed by the Cell no_agg operator of the Cell listing."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(51)
    m, n, r = 300, 200, 20
    rp, ci, va = W.csr_bernoulli(m, n, 0.05, 52)
    x = ops.make_csr(rp, ci, va, (m, n))
    u, v, rr = rng.uniform(size=(m, r)), rng.uniform(size=(n, r)), rng.uniform(size=m)
    inner = F.fuse_outer(ALS_W, dev_csr(rp, ci, va, (m, n)), to_dev(u), to_dev(v), [], "right_mm").view(m, r)
    cell = [("side", 0), ("main",), ("const", 1e-6), ("mul",), ("side", 1), ("mul",), ("add",)]   # I + U*1e-6*r
    got = host(F.fuse_cell(cell, to_dev(u), [("matrix", inner), ("colvec", to_dev(rr))], "none")).reshape(m, r)
    ref_inner = unfused.outer(ALS_W, x, u, v, [], "right_mm")
    ref = unfused.cell(cell, u, [("matrix", ref_inner), ("colvec", rr)], "none")
    assert_close(got, ref, what="ALS-CG update")
    d = ops.csr_to_dense(x)
    np.testing.assert_allclose(got, ((d != 0) * (u @ v.T)) @ v + 1e-6 * u * rr[:, None], rtol=1e-11)


@pytest.mark.parametrize("nops", [1, 8, 40, 300])
def test_row_long_chain_expression(nops):
    """sum(f(X / rowSums(X))) with f a chain of `nops` scalar multiplications (the expression of
    the instruction-footprint experiment, Sec. 5.2): one reduction stage, then a long body."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(61)
    m, n = 257, 1000
    x = rng.uniform(0.5, 1.5, size=(m, n))
    expr = [("main",), ("main",), ("rowsum",), ("div",)]
    for i in range(1, nops + 1):
        expr += [("const", 1.0 + 1.0 / (i + 1)), ("mul",)]
    got = host(F.fuse_row(expr, to_dev(x), [], "full"))
    assert_close(got, unfused.row_dense(expr, x, [], "full"), what="chain %d" % nops)
    got = host(F.fuse_row(expr, to_dev(x), [], "none"))
    assert_close(got, unfused.row_dense(expr, x, [], "none"), what="chain %d none" % nops)


# ------------------------------------------------- Cell / MAgg over a sparse X ---

@pytest.mark.parametrize("case", range(10 * MORE))
def test_sparse_cell_and_magg_random_expressions(case, csr_mapping):
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(9700 + case)
    m, n = [(1, 1), (37, 19), (300, 1000), (1000, 100), (64, 3000)][case % 5]
    dens = [1.0, 0.3, 0.1, 0.02, 0.004][case % 5]
    rp, ci, va = W.csr_bernoulli(m, n, dens, 9700 + case)
    x = ops.make_csr(rp, ci, va, (m, n))
    sides = _sides(rng, m, n)
    xd, sd = dev_csr(rp, ci, va, (m, n)), dev_sides(sides)
    exprs = [random_row_expr(rng, KINDS, depth=3, want="V", sparse_safe=True, reductions=False) for _ in range(3)]
    for agg in ("none", "row", "col", "full"):
        print("sparse cell case", case, (m, n), agg, exprs[0], flush=True)
        got = host(F.fuse_cell_csr(exprs[0], xd, sd, agg))
        ref = unfused.cell_csr(exprs[0], x, sides, agg)
        a = np.abs(np.nan_to_num(unfused.cell_csr(exprs[0], x, sides, "none"), nan=0, posinf=0, neginf=0))
        scale = {"none": None, "full": a.sum(), "row": ops.csr_row_sums(x, a).max(initial=0.0),
                 "col": ops.csr_col_sums(x, a).max(initial=0.0)}[agg]
        assert_close(got, ref, scale=None if scale is None else max(scale, 1e-300), what="sparse cell %s" % agg)
    got = host(F.fuse_magg_csr(exprs, xd, sd))
    ref = unfused.magg_csr(exprs, x, sides)
    for j in range(3):
        a = np.abs(np.nan_to_num(unfused.cell_csr(exprs[j], x, sides, "none"), nan=0, posinf=0, neginf=0))
        assert_close(got[j], ref[j], scale=max(a.sum(), 1e-300), what="sparse magg[%d]" % j)
        one = host(F.fuse_cell_csr(exprs[j], xd, sd, "full"))
        assert_close(got[j], one[0], scale=max(a.sum(), 1e-300), tol=1e-13, what="sparse magg vs cell [%d]" % j)


def test_sparse_cell_paper_expression_and_rejections(csr_mapping):
    """sum(X * Y * Z) with a sparse X (density 0.1) and dense Y, Z: equals the dense operator
    on the densified X; bodies that are not sparse-safe are rejected."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(81)
    m, n = 2000, 1000
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 82)
    y, z = rng.uniform(size=(2, m, n))
    xd = dev_csr(rp, ci, va, (m, n))
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    sd = [("matrix", to_dev(y)), ("matrix", to_dev(z))]
    got = host(F.fuse_cell_csr(expr, xd, sd, "full"))
    dense = ops.csr_to_dense(ops.make_csr(rp, ci, va, (m, n)))
    from oracle import plans
    assert_close(got, plans.cell_sum_xyz(dense, y, z), what="sparse sum(XYZ)")
    assert_close(got, host(F.fuse_cell(expr, to_dev(dense), sd, "full")), tol=1e-12, what="sparse vs dense operator")
    for bad in ([("main",), ("const", 1.0), ("add",)], [("side", 0)]):
        with pytest.raises(F.FuseError) as e:
            F.fuse_cell_csr(bad, xd, sd, "full")
        assert e.value.code == -3


# ------------------------------------------------------- sparse side inputs ---

def _sparse_side(m, n, dens, seed, rowptr64=False):
    """A CSR side input for the GPU and the same matrix densified for the oracle (whose operators take the side
    as the matrix it is: a value per cell, 0 where nothing is stored)."""
    rp, ci, va = W.csr_bernoulli(m, n, dens, seed)
    dense = ops.csr_to_dense(ops.make_csr(rp, ci, va, (m, n))) if m * n else np.zeros((m, n))
    return ("sparse", (rp, ci, va, (m, n), rowptr64)), ("matrix", dense)


@pytest.mark.parametrize("case", range(5 * MORE))
def test_sparse_side_inputs_random_expressions(case, csr_mapping):
    """Cell, MAgg and Row bodies over a CSR main input whose matrix side input is sparse as well (Table 1: sparse /
    dense side inputs; Fig. 8b / 8d): every result against the oracle's operator-at-a-time plan on the densified side."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(9900 + case)
    m, n = [(1, 1), (37, 19), (300, 1000), (1000, 100), (64, 3000)][case % 5]
    dens = [1.0, 0.3, 0.1, 0.02, 0.004][case % 5]
    sdens = [1.0, 0.5, 0.1, 0.3, 0.01][(case + 2) % 5]
    rp, ci, va = W.csr_bernoulli(m, n, dens, 9900 + case)
    x = ops.make_csr(rp, ci, va, (m, n))
    gpu_side, ref_side = _sparse_side(m, n, sdens, 19900 + case, rowptr64=bool(case % 2))
    rest = _sides(rng, m, n)[1:]
    sides, gsides = [ref_side] + rest, [gpu_side] + rest
    xd, sd = dev_csr(rp, ci, va, (m, n)), dev_sides(gsides)
    exprs = [random_row_expr(rng, KINDS, depth=3, want="V", sparse_safe=True, reductions=False) for _ in range(3)]
    exprs[0] = [("main",), ("side", 0), ("mul",)] + exprs[0] + [("mul",)]          # the sparse side is in every run
    for agg in ("none", "row", "col", "full"):
        print("sparse side cell case", case, (m, n), agg, exprs[0], flush=True)
        got = host(F.fuse_cell_csr(exprs[0], xd, sd, agg))
        ref = unfused.cell_csr(exprs[0], x, sides, agg)
        a = np.abs(np.nan_to_num(unfused.cell_csr(exprs[0], x, sides, "none"), nan=0, posinf=0, neginf=0))
        scale = {"none": None, "full": a.sum(), "row": ops.csr_row_sums(x, a).max(initial=0.0),
                 "col": ops.csr_col_sums(x, a).max(initial=0.0)}[agg]
        assert_close(got, ref, scale=None if scale is None else max(scale, 1e-300), what="sparse side cell %s" % agg)
    got = host(F.fuse_magg_csr(exprs, xd, sd))
    ref = unfused.magg_csr(exprs, x, sides)
    for j in range(3):
        a = np.abs(np.nan_to_num(unfused.cell_csr(exprs[j], x, sides, "none"), nan=0, posinf=0, neginf=0))
        assert_close(got[j], ref[j], scale=max(a.sum(), 1e-300), what="sparse side magg[%d]" % j)
    # a Row body with row aggregates
    expr = [("main",), ("side", 0), ("mul",)] + random_row_expr(rng, KINDS, depth=3, want="V", sparse_safe=True) + [("mul",)]
    none_ref = unfused.row_csr(expr, x, sides, "none")
    a = np.abs(np.nan_to_num(none_ref, nan=0.0, posinf=0.0, neginf=0.0))
    for agg in ("none", "row", "col_t", "full"):
        print("sparse side row case", case, (m, n), agg, expr, flush=True)
        got = host(F.fuse_row(expr, xd, sd, agg))
        ref = unfused.row_csr(expr, x, sides, agg)
        scale = {"none": None, "full": a.sum(), "row": ops.csr_row_sums(x, a).max(initial=0.0),
                 "col_t": ops.csr_col_sums(x, a).max(initial=0.0)}[agg]
        assert_close(got, ref, scale=None if scale is None else max(scale, 1e-300), what="sparse side row %s" % agg)


def test_sparse_side_inputs_paper_expression_and_rejections(csr_mapping):
    """sum(X * Y * Z) with X, Y and Z sparse (Fig. 8b; density 0.1): the oracle's plan on the densified matrices, the
    dense-side operator on the same values, and the calls that do not take a sparse side."""
    import paper_1801_00829_amd as F
    from oracle import plans
    m, n = 2000, 1000
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 91)
    (ky, ysp), (_, yd) = _sparse_side(m, n, 0.1, 92)
    (kz, zsp), (_, zd) = _sparse_side(m, n, 0.1, 93, rowptr64=True)
    xd = dev_csr(rp, ci, va, (m, n))
    expr = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]
    sd = dev_sides([(ky, ysp), (kz, zsp)])
    dense = ops.csr_to_dense(ops.make_csr(rp, ci, va, (m, n)))
    got = host(F.fuse_cell_csr(expr, xd, sd, "full"))
    assert_close(got, plans.cell_sum_xyz(dense, yd, zd), scale=np.abs(dense * yd * zd).sum(), what="sum(XYZ), all sparse")
    dsd = [("matrix", to_dev(yd)), ("matrix", to_dev(zd))]
    assert_close(got, host(F.fuse_cell_csr(expr, xd, dsd, "full")), tol=1e-12, what="sparse against dense sides")
    two = host(F.fuse_magg_csr([expr[:3], [("main",), ("side", 1), ("mul",)]], xd, sd))
    assert_close(two[0], (dense * yd).sum(), scale=np.abs(dense * yd).sum(), what="sum(XY), sparse")
    assert_close(two[1], (dense * zd).sum(), scale=np.abs(dense * zd).sum(), what="sum(XZ), sparse")
    # an empty side: every product is zero
    empty = ("sparse", (np.zeros(m + 1, np.int64), np.zeros(0, np.int32), np.zeros(0), (m, n)))
    assert host(F.fuse_cell_csr(expr, xd, dev_sides([empty, (kz, zsp)]), "full"))[0] == 0.0
    # calls that bind to dense side inputs only
    with pytest.raises(F.FuseError) as e:
        F.fuse_cell(expr, to_dev(dense), sd, "full")
    assert e.value.code == -7
    u = to_dev(np.ones((m, 3)))
    v = to_dev(np.ones((n, 3)))
    with pytest.raises(F.FuseError) as e:
        F.fuse_outer([("main",), ("uvdot",), ("mul",), ("side", 0), ("mul",)], xd, u, v, sd[:1], "full")
    assert e.value.code == -7
    with pytest.raises(F.FuseError) as e:
        F.fuse_row(expr, to_dev(dense), sd, "full")
    assert e.value.code == -7
    wrong = dev_sides([_sparse_side(m, n + 1, 0.1, 94)[0]])
    with pytest.raises(F.FuseError) as e:
        F.fuse_cell_csr(expr[:3], xd, wrong, "full")
    assert e.value.code == -2


@pytest.mark.parametrize("scap", ["0", "8", "64"])
def test_sparse_side_lookup_paths_agree(scap, monkeypatch):
    """The three ways a cell finds its value in a sparse side -- the side's row staged in LDS, a side row too long for
    its LDS slot, every look-up in memory -- against the oracle and against each other (lane-group kernel)."""
    import paper_1801_00829_amd as F
    monkeypatch.setenv("FUSE_CSR_STREAM", "0")
    monkeypatch.setenv("FUSE_CSR_SCAP", scap)
    m, n = 4000, 500
    rp, ci, va = W.csr_bernoulli(m, n, 0.08, 95)
    x = ops.make_csr(rp, ci, va, (m, n))
    (ky, ysp), ref_y = _sparse_side(m, n, 0.06, 96)                      # ~30 cells per row: over 8, under 64
    (kz, zsp), ref_z = _sparse_side(m, n, 0.2, 97, rowptr64=True)        # ~100 cells per row: over both
    xd = dev_csr(rp, ci, va, (m, n))
    sd = dev_sides([(ky, ysp), (kz, zsp)])
    expr = [("main",), ("side", 0), ("mul",), ("main",), ("side", 1), ("mul",), ("add",)]        # X*Y + X*Z
    for agg in ("none", "row", "col", "full"):
        got = host(F.fuse_cell_csr(expr, xd, sd, agg))
        ref = unfused.cell_csr(expr, x, [ref_y, ref_z], agg)
        a = np.abs(unfused.cell_csr(expr, x, [ref_y, ref_z], "none"))
        scale = {"none": None, "full": a.sum(), "row": ops.csr_row_sums(x, a).max(initial=0.0),
                 "col": ops.csr_col_sums(x, a).max(initial=0.0)}[agg]
        assert_close(got, ref, scale=scale, what="sparse sides, %s LDS entries, %s" % (scap, agg))
    assert ("#define FUSE_SCAP %s\n" % scap) in F.last_source()


# ------------------------------------------- Row with a matrix right-hand side ---

MLOG_Q = [("side", 1), ("main",), ("side", 0), ("matmult",), ("mul",)]                   # Q = P * (X V)
MLOGREG = [("main",)] + MLOG_Q + [("side", 1)] + MLOG_Q + [("rowsum",), ("mul",), ("sub",), ("outerk",)]
TXXV = [("main",), ("main",), ("side", 0), ("matmult",), ("outerk",)]                     # t(X) (X V)


@pytest.fixture(params=["vector", "matrix_units", "matrix_units_blocks"])
def rhs_form(request, monkeypatch):
    """The forms of t(X) (f(X V)) bodies: k-vectors on the vector ALUs (k butterflies per row), or the
    two products on the fp64 matrix units (by default from 3 or 5 classes on, while 16 rows fit in LDS):
    one wave per 16-row tile for contiguous matrices of at most 112 columns, a block per tile otherwise
    ("matrix_units_blocks" takes the block form for the narrow matrices too)."""
    monkeypatch.setenv("FUSE_MFMA_MIN_K", "0" if request.param == "vector" else "1")
    if request.param == "matrix_units_blocks":
        monkeypatch.setenv("FUSE_MFMA_WAVE_FORM", "0")
    return request.param


@pytest.mark.parametrize("shape", [(1, 1, 1), (70, 10, 3), (333, 100, 4), (129, 101, 2), (64, 1000, 2), (50, 784, 1),
                                   (500, 37, 16), (120, 784, 10), (33, 2048, 16), (40, 1000, 8), (17, 4096, 5), (9, 3000, 3),
                                   (4100, 17, 7), (16, 16, 16), (15, 1199, 2), (70001, 100, 6), (40003, 29, 9), (35000, 112, 16)])
def test_row_matrix_rhs_chain_and_mlogreg_core(shape, rhs_form):
    """t(X) %*% (X %*% V) with an n x k right-hand side (Fig. 8g) and the multinomial logistic
    regression core H = t(X) (Q - P * rowSums(Q)), Q = P * (X V)  (Sec. 2.2, second example)."""
    import paper_1801_00829_amd as F
    from oracle import plans
    m, n, k = shape
    rng = np.random.default_rng(71)
    x, v, p = rng.normal(size=(m, n)), rng.normal(size=(n, k)), rng.uniform(size=(m, k))
    xd, vd, pd = to_dev(x), to_dev(v), to_dev(p)
    sd = [("rhs", vd), ("kvec", pd)]
    print("row matrix rhs", shape, flush=True)
    absx, absv = np.abs(x), np.abs(v)
    scale = max((absx.T @ (absx @ absv)).max(), 1e-300)
    got = host(F.fuse_row(TXXV, xd, sd, "col_t")).reshape(n, k)
    assert_close(got, plans.row_tx_xv_matrix(x, v), scale=scale, what="t(X)(XV)")
    if 16 <= n <= 1000:
        assert F.last_kernel().startswith("fuse_row_mfma_") == (rhs_form != "vector")
        if n <= 112:
            assert F.last_kernel().startswith("fuse_row_mfma_wave_") == (rhs_form == "matrix_units")
    got = host(F.fuse_row(MLOGREG, xd, sd, "col_t")).reshape(n, k)
    assert_close(got, plans.mlogreg_core(x, v, p), scale=2 * k * scale, what="mlogreg core")
    assert_close(got, unfused.row_dense(MLOGREG, x, [("rhs", v), ("kvec", p)], "col_t"), scale=2 * k * scale,
                 what="mlogreg core vs generic evaluator")
    # k-vector results: X V (no_agg), its column sums, its total; rowSums(Q) per row
    xv = [("main",), ("side", 0), ("matmult",)]
    s1 = max((absx @ absv).max(), 1e-300)
    assert_close(host(F.fuse_row(xv, xd, sd, "none")).reshape(m, k), x @ v, scale=s1, what="X V")
    assert_close(host(F.fuse_row(xv, xd, sd, "col")), unfused.row_dense(xv, x, [("rhs", v)], "col"),
                 scale=(absx @ absv).sum(0).max(), what="colSums(X V)")
    assert_close(host(F.fuse_row(xv, xd, sd, "full")), unfused.row_dense(xv, x, [("rhs", v)], "full"),
                 scale=(absx @ absv).sum(), what="sum(X V)")
    assert_close(host(F.fuse_row(MLOG_Q + [("rowsum",)], xd, sd, "none")),
                 unfused.row_dense(MLOG_Q + [("rowsum",)], x, [("rhs", v), ("kvec", p)], "none"),
                 scale=(absx @ absv).sum(1).max(), what="rowSums(Q)")


@pytest.mark.parametrize("k", [1, 3, 10, 16])
def test_row_csr_matrix_rhs_on_all_patterns(k):
    """t(X)(XV), the MLogreg core and k-vector results over a CSR main input: products over the stored
    cells of a row (vectMatMult), outer products summed into n x k (vectOuterMultAdd)."""
    import paper_1801_00829_amd as F
    xv = [("main",), ("side", 0), ("matmult",)]
    for name, (rp, ci, va), shape in _csr_cases():
        m, n = shape
        rng = np.random.default_rng(91)
        v, p = rng.normal(size=(n, k)), rng.uniform(size=(m, k))
        x = ops.make_csr(rp, ci, va, shape)
        xd, sd = dev_csr(rp, ci, va, shape), [("rhs", to_dev(v)), ("kvec", to_dev(p))]
        hs = [("rhs", v), ("kvec", p)]
        print("row csr matrix rhs", name, shape, "k", k, flush=True)
        ax = ops.make_csr(rp, ci, np.abs(va), shape)
        absq = ops.csr_matmul_dense(ax, ax.vals, np.abs(v)) if va.size else np.zeros((m, k))
        scale = max(ops.csr_t_matmul_dense(ax, ax.vals, absq).max(initial=0.0), 1e-300)
        for expr, fac in ((TXXV, 1.0), (MLOGREG, 2.0 * k)):
            got = host(F.fuse_row(expr, xd, sd, "col_t")).reshape(n, k)
            ref = unfused.row_csr(expr, x, hs, "col_t")
            assert_close(got, ref, scale=fac * scale, what="csr %s" % ("t(X)(XV)" if expr is TXXV else "mlogreg core"))
            assert not got[np.bincount(ci, minlength=n) == 0].any()          # columns without stored cells
        s1 = max(absq.max(initial=0.0), 1e-300)
        got = host(F.fuse_row(xv, xd, sd, "none")).reshape(m, k)
        assert_close(got, unfused.row_csr(xv, x, hs, "none"), scale=s1, what="csr X V")
        assert not got[np.diff(rp) == 0].any()                               # rows without stored cells
        assert_close(host(F.fuse_row(xv, xd, sd, "col")), unfused.row_csr(xv, x, hs, "col"),
                     scale=max(absq.sum(0).max(initial=0.0), 1e-300), what="csr colSums(X V)")
        assert_close(host(F.fuse_row(xv, xd, sd, "full")), unfused.row_csr(xv, x, hs, "full"),
                     scale=max(absq.sum(), 1e-300), what="csr sum(X V)")
        # a body that also has a value on rows without stored cells: rowSums(P * (X V)) + rowSums(P)
        e2 = MLOG_Q + [("rowsum",), ("side", 1), ("rowsum",), ("add",)]
        assert_close(host(F.fuse_row(e2, xd, sd, "none")), unfused.row_csr(e2, x, hs, "none"),
                     scale=max(absq.sum(1).max(initial=0.0) + k, 1.0), what="csr rowSums(Q) + rowSums(P)")


@pytest.mark.parametrize("rowptr64", [False, True])
@pytest.mark.parametrize("case", ["mnist_like", "skewed", "narrow_full", "ragged_tail"])
def test_row_csr_matrix_rhs_through_the_matrix_units(case, rowptr64, monkeypatch):
    """CSR matrices that store a good part of their cells (Mnist-like: a quarter) take the dense matrix-unit
    form, whose LDS tile is filled from the CSR rows: rows longer and shorter than what travels in registers,
    empty rows, a row count that is no multiple of the tile; against the oracle's evaluation over the stored
    cells and against the lane-group form."""
    import torch
    import paper_1801_00829_amd as F
    if case == "mnist_like":
        shape, k = (3001, 784), 10
        rp, ci, va = W.csr_bernoulli(*shape, 0.25, 301)
    elif case == "skewed":                       # most rows 16 % full, a few 95 % full, every seventh empty
        shape, k = (1500, 300), 7
        rp, ci, va = W.csr_skewed(*shape, 0.16, 40, 0.95, 302)
        lens = np.diff(rp)
        keep_row = np.arange(shape[0]) % 7 != 0
        keep = np.repeat(keep_row, lens)
        rp2 = np.zeros(shape[0] + 1, np.int64)
        np.cumsum(np.where(keep_row, lens, 0), out=rp2[1:])
        rp, ci, va = rp2, ci[keep], va[keep]
    elif case == "narrow_full":
        shape, k = (4100, 17), 16
        rp, ci, va = W.csr_bernoulli(*shape, 1.0, 303)
    else:
        shape, k = (33, 1100), 5
        rp, ci, va = W.csr_bernoulli(*shape, 0.5, 304)
    m, n = shape
    rng = np.random.default_rng(92)
    v, p = rng.normal(size=(n, k)), rng.uniform(size=(m, k))
    x = ops.make_csr(rp, ci, va, shape)
    rpd = torch.from_numpy(rp).to(torch.int64 if rowptr64 else torch.int32).cuda()
    xd = F.Csr(rpd, torch.from_numpy(ci).cuda(), to_dev(va), shape)
    sd, hs = [("rhs", to_dev(v)), ("kvec", to_dev(p))], [("rhs", v), ("kvec", p)]
    ax = ops.make_csr(rp, ci, np.abs(va), shape)
    absq = ops.csr_matmul_dense(ax, ax.vals, np.abs(v))
    scale = max(ops.csr_t_matmul_dense(ax, ax.vals, absq).max(initial=0.0), 1e-300)
    for expr, fac in ((TXXV, 1.0), (MLOGREG, 2.0 * k)):
        print("row csr matrix units", case, shape, "k", k, "rowptr64", rowptr64, flush=True)
        got = host(F.fuse_row(expr, xd, sd, "col_t")).reshape(n, k)
        assert F.last_kernel().startswith("fuse_row_mfma_")
        ref = unfused.row_csr(expr, x, hs, "col_t")
        assert_close(got, ref, scale=fac * scale, what="csr matrix units")
        monkeypatch.setenv("FUSE_MFMA_CSR_MIN_K", "0")
        other = host(F.fuse_row(expr, xd, sd, "col_t")).reshape(n, k)
        assert F.last_kernel().startswith("fuse_row_csr_")
        monkeypatch.delenv("FUSE_MFMA_CSR_MIN_K")
        assert_close(got, other, scale=fac * scale, what="csr matrix units against lane groups")


def test_row_matrix_rhs_strided_sides_and_limits(rhs_form):
    import paper_1801_00829_amd as F
    from oracle import plans
    rng = np.random.default_rng(72)
    m, n, k = 200, 50, 3
    xb = rng.normal(size=(m, n + 3))
    x = xb[:, :n]
    # a view of X with a leading dimension > cols and an odd column count elsewhere
    got = host(F.fuse_row(TXXV, to_dev(xb)[:, :n], [("rhs", to_dev(rng.normal(size=(n, k))))], "col_t"))
    assert got.size == n * k
    vb, pb = rng.normal(size=(n, k + 2)), rng.uniform(size=(m, k + 5))
    v, p = vb[:, 1:1 + k], pb[:, 2:2 + k]
    got = host(F.fuse_row(MLOGREG, to_dev(x), [("rhs", to_dev(vb)[:, 1:1 + k]), ("kvec", to_dev(pb)[:, 2:2 + k])],
                          "col_t")).reshape(n, k)
    assert_close(got, plans.mlogreg_core(x, v, p), scale=np.abs(x).T @ (np.abs(x) @ np.abs(v)) * 2 * k, what="strided rhs")
    import torch
    with pytest.raises(F.FuseError) as e:       # too many columns x k for the register-resident form
        F.fuse_row(TXXV, torch.ones((4, 6000), dtype=torch.float64, device="cuda"),
                   [("rhs", torch.ones((6000, 16), dtype=torch.float64, device="cuda"))], "col_t")
    assert e.value.code == -7
    with pytest.raises(F.FuseError) as e:       # shapes: the right-hand side must have cols(X) rows
        F.fuse_row(TXXV, to_dev(x), [("rhs", to_dev(np.ones((n + 1, k))))], "col_t")
    assert e.value.code == -2


# ------------------------------------------------------------ more edge cases ---

def test_zero_sized_inputs_everywhere():
    """Matrices without rows, without columns or without stored cells through every entry point: zero
    sums, empty outputs, no launch on empty grids."""
    import torch
    import paper_1801_00829_amd as F
    z = lambda *shape: torch.zeros(shape, dtype=torch.float64, device="cuda")
    dot = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    for m, n in ((0, 7), (5, 0), (0, 0)):
        x = z(m, n)
        assert host(F.fuse_cell([("main",)], x, [], "full")).tolist() == [0.0]
        assert host(F.fuse_cell([("main",)], x, [], "row")).tolist() == [0.0] * m
        assert host(F.fuse_cell([("main",)], x, [], "col")).tolist() == [0.0] * n
        assert host(F.fuse_cell([("main",)], x, [], "none")).size == 0
        assert host(F.fuse_magg([[("main",)], [("main",), ("pow2",)]], x, [])).tolist() == [0.0, 0.0]
        assert host(F.fuse_row(dot, x, [("rowvec", z(n))], "col_t")).tolist() == [0.0] * n
        assert host(F.fuse_row([("main",), ("rowsum",)], x, [], "none")).tolist() == [0.0] * m
        # the same shapes as CSR without stored cells
        xs = F.Csr(torch.zeros(m + 1, dtype=torch.int32, device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"),
                   z(0), (m, n))
        F.check_csr(xs)
        for form in ("0", "1"):
            import os
            os.environ["FUSE_CSR_STREAM"] = form
            try:
                assert host(F.fuse_row(dot, xs, [("rowvec", z(n))], "col_t")).tolist() == [0.0] * n
                assert host(F.fuse_row([("main",)], xs, [], "row")).tolist() == [0.0] * m
                assert host(F.fuse_row([("main",)], xs, [], "full")).tolist() == [0.0]
                assert host(F.fuse_row([("main",)], xs, [], "none")).size == 0
                assert host(F.fuse_cell_csr([("main",), ("pow2",)], xs, [], "full")).tolist() == [0.0]
                assert host(F.fuse_magg_csr([[("main",)], [("main",), ("abs",)]], xs, [])).tolist() == [0.0, 0.0]
            finally:
                os.environ.pop("FUSE_CSR_STREAM", None)
        r = 3
        for agg, count in (("full", 1), ("none", 0), ("right_mm", m * r), ("left_mm", n * r)):
            got = host(F.fuse_outer([("main",), ("uvdot",), ("mul",)], xs, z(m, r), z(n, r), [], agg))
            assert got.size == count and not got.any(), (m, n, agg)


def test_row_body_with_the_most_reductions_and_stages():
    """64 row aggregates in one stage (the most a body may have; 65 are rejected), and five nested stages."""
    import paper_1801_00829_amd as F
    rng = np.random.default_rng(71)
    m, n = 150, 130
    x = rng.uniform(0.5, 1.5, size=(m, n))
    body = [("main",), ("const", 1.0), ("mul",), ("rowsum",)]
    for i in range(2, 65):
        body += [("main",), ("const", float(i)), ("mul",), ("rowsum",), ("add",)]
    got = host(F.fuse_row(body, to_dev(x), [], "none"))
    assert_close(got, unfused.row_dense(body, x, [], "none"), what="64 reductions")
    rp, ci, va = W.csr_bernoulli(m, n, 0.1, 72)
    got = host(F.fuse_row(body, dev_csr(rp, ci, va, (m, n)), [], "none"))
    assert_close(got, unfused.row_csr(body, ops.make_csr(rp, ci, va, (m, n)), [], "none"), what="64 reductions, CSR")
    with pytest.raises(F.FuseError):
        F.fuse_row(body + [("main",), ("const", 65.0), ("mul",), ("rowsum",), ("add",)], to_dev(x), [], "none")
    # five stages: s1 = rowsum(X); s2 = rowsum(X / s1); s3 = rowsum(X * s2) ...
    nested = [("main",), ("rowsum",)]
    for i in range(4):
        nested = [("main",)] + nested + [("div",) if i % 2 == 0 else ("mul",), ("rowsum",)]
    for agg in ("none", "full"):
        got = host(F.fuse_row(nested, to_dev(x), [], agg))
        assert_close(got, unfused.row_dense(nested, x, [], agg), tol=1e-10, what="five stages " + agg)
    assert "#define FUSE_NSTAGE 5" in F.last_source()


def test_code_object_from_the_cache_directory_runs(tmp_path, monkeypatch):
    """A body compiled in an earlier life of the in-memory plan cache is loaded from FUSE_CACHE_DIR and
    gives the same bits."""
    import paper_1801_00829_amd as F
    monkeypatch.setenv("FUSE_CACHE_DIR", str(tmp_path))
    rng = np.random.default_rng(99)
    x, y = rng.normal(size=(2, 300, 77))
    v = rng.normal(size=77)
    cell = [("main",), ("side", 0), ("mul",), ("const", 0.987654321), ("add",), ("abs",)]
    row = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    xd, yd, vd = to_dev(x), to_dev(y), to_dev(v)
    F.cache_clear()
    first = host(F.fuse_cell(cell, xd, [("matrix", yd)], "full")), host(F.fuse_row(row, xd, [("rowvec", vd)], "col_t"))
    assert F.cache_disk_hits() == 0 and len(os.listdir(tmp_path)) == 2
    F.cache_clear()
    again = host(F.fuse_cell(cell, xd, [("matrix", yd)], "full")), host(F.fuse_row(row, xd, [("rowvec", vd)], "col_t"))
    assert F.cache_disk_hits() == 2 and F.cache_stats()[2] == 0.0
    assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])
    assert_close(again[0], unfused.cell(cell, x, [("matrix", y)], "full"), scale=np.abs(x * y + 0.987654321).sum(), what="cached cell")
    F.cache_clear()
