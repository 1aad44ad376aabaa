"""Host-side checks of libfuse without a GPU: exported symbols, validation and
error codes, descriptor type checking, hipRTC compilation of generated bodies
for gfx950 (hipRTC needs no device), plan-cache behaviour."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def F():
    import paper_1801_00829_amd as F
    from paper_1801_00829_amd import build as B
    if B.needs_build():
        B.build()
    return F


def test_library_exports_every_declared_symbol(F):
    hdr = open(os.path.join(ROOT, "include", "fuse.h")).read()
    declared = set(re.findall(r"^(?:int|int64_t|void|size_t|const char \*)\s*\*?(fuse_\w+)\(", hdr, flags=re.M))
    assert {"fuse_cell", "fuse_magg", "fuse_row", "fuse_outer", "fuse_last_error", "fuse_cache_stats",
            "fuse_cache_clear", "fuse_prepare_cell", "fuse_prepare_magg", "fuse_prepare_row",
            "fuse_prepare_outer", "fuse_last_source", "fuse_last_kernel", "fuse_probe_copy",
            "fuse_probe_read", "fuse_cache_disk_hits", "fuse_check_csr", "fuse_magg_noalloc", "fuse_row_out_count",
            "fuse_probe_gather"} <= declared
    lib = ctypes.CDLL(F.lib_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_binding_opcodes_match_header(F):
    hdr = open(os.path.join(ROOT, "include", "fuse.h")).read()
    body = hdr[hdr.index("typedef enum {\n    /* leaves */"):hdr.index("} fuse_op;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    val, enum = -1, {}
    for item in body.replace("typedef enum {", "").split(","):
        item = item.strip()
        if not item:
            continue
        if "=" in item:
            name, v = [t.strip() for t in item.split("=")]
            val = int(v)
        else:
            name, val = item, val + 1
        enum[name] = val
    for name, code in F.OPS.items():
        assert enum["FUSE_OP_" + name.upper()] == code, name


XYZ = [("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]


def test_prepare_compiles_the_five_workloads_and_caches(F):
    F.cache_clear()
    two = [("matrix", None), ("matrix", None)]
    F.prepare_cell(XYZ, (1000, 1000), two, "full")
    assert F.last_kernel().startswith("fuse_cell_")
    src = F.last_source()
    assert re.search(r"const double (v\d+_0) = a \* s\[0\];\s+const double (v\d+_0) = \1 \* s\[1\];\s+r\[0\] = \2;", src)
    assert "fuse_grid_finish" in src
    F.prepare_magg([XYZ[:3], [("main",), ("side", 1), ("mul",)], [("main",), ("pow2",)]], (100000, 1000), two)
    assert re.search(r"const double (v\d+_0) = fuse_pow2\(a\);\s+r\[2\] = \1;", F.last_source())
    F.prepare_row([("main",), ("side", 0), ("dot",), ("side", 1), ("mul",), ("main",), ("mul",)], (1000000, 100),
                  [("rowvec", None), ("colvec", None)], "col_t")
    src = F.last_source()
    assert "part[0] += a * sv[0];" in src
    assert re.search(r"const double (v\d+_0) = red\[0\] \* rsc\[1\];\s+const double (v\d+_0) = \1 \* a;\s+return \2;", src)
    assert "#define FUSE_G 16" in src and "#define FUSE_EPL 4" in src and "#define FUSE_VEC 2" in src
    F.prepare_row([("main",), ("side", 0), ("dot",), ("main",), ("mul",)], (10000000, 1000), [("rowvec", None)],
                  "col_t", nnz=100000000)
    assert F.last_kernel().startswith("fuse_row_csr_") and "#define FUSE_C " in F.last_source()
    F.prepare_outer([("main",), ("uvdot",), ("const", 1e-15), ("add",), ("log",), ("mul",)], (100000, 100000), 100,
                    10000000)
    assert re.search(r"const double (v\d+_0) = d \+ \(0x1\.203af9ee75616p-50\);\s+const double (v\d+_0) = log\(\1\);\s+"
                     r"const double (v\d+_0) = a \* \2;\s+return \3;", F.last_source())
    hits, misses, ms = F.cache_stats()
    assert (hits, misses) == (0, 5) and ms > 0
    # equal descriptors are compiled once (plan cache)
    F.prepare_cell(XYZ, (1000, 1000), two, "full")
    F.prepare_cell(XYZ, (123, 77), two, "full")          # the shape is not part of a flat Cell plan
    assert F.cache_stats()[:2] == (2, 5)
    F.prepare_cell(XYZ, (1000, 1000), two, "none")       # another variant is another plan
    assert F.cache_stats()[:2] == (2, 6)


def test_constants_round_trip_exactly(F):
    for c in (1e-15, 0.1, -2.5e300, 5e-324):
        F.prepare_cell([("main",), ("const", c), ("add",)], (4, 4), [], "full")
        lit = re.search(r"= a \+ \((-?0x[0-9a-fp.+-]+)\);", F.last_source()).group(1)
        assert float.fromhex(lit) == c


@pytest.mark.parametrize("expr,code", [
    ([("main",), ("mul",)], -3),                              # binary operator with one operand
    ([("main",), ("main",)], -3),                             # two values left on the stack
    ([("main",), ("side", 5), ("mul",)], -3),                 # side index out of range
    ([("main",), ("rowsum",)], -3),                           # row token in a Cell body
    ([("uvdot",)], -3),                                       # Outer token in a Cell body
    ([], -1),                                                 # empty expression
])
def test_cell_descriptor_errors(F, expr, code):
    with pytest.raises(F.FuseError) as e:
        F.prepare_cell(expr, (8, 8), [("matrix", None)], "full")
    assert e.value.code == code
    assert str(e.value)


def test_shape_and_argument_errors(F):
    from paper_1801_00829_amd import _lib as L
    lib = L.load()
    e, keep = F.api._expr(XYZ)
    x = L.Dense(None, 8, 8, 8)
    sides = (L.Side * 2)()
    sides[0].kind, sides[0].m = 0, L.Dense(None, 8, 9, 9)      # wrong shape
    sides[1].kind, sides[1].m = 0, L.Dense(None, 8, 8, 8)
    assert lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(x), sides, 2, 1) == -2
    assert b"side 0" in lib.fuse_last_error()
    sides[0].m = L.Dense(None, 8, 8, 4)                        # ld < cols
    assert lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(x), sides, 2, 1) == -2
    sides[0].m = L.Dense(None, 8, 8, 8)
    assert lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(x), sides, 2, 9) == -1     # bad aggregation
    assert lib.fuse_prepare_cell(None, ctypes.byref(x), sides, 2, 1) == -1
    assert lib.fuse_prepare_cell(ctypes.byref(e), None, sides, 2, 1) == -1
    assert lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(x), sides, 9, 1) == -1     # too many sides
    assert lib.fuse_prepare_cell(ctypes.byref(e), ctypes.byref(x), sides, 2, 1) == 0
    assert lib.fuse_last_error() == b""
    # launching calls reject NULL data / out before touching the device
    assert lib.fuse_cell(ctypes.byref(e), ctypes.byref(x), sides, 2, 1, None, None) == -1
    # Row: exactly one main input
    xs = L.CsrDesc(None, None, None, 0, 8, 8, 10)
    assert lib.fuse_prepare_row(ctypes.byref(e), ctypes.byref(x), ctypes.byref(xs), sides, 2, 3) == -1
    assert lib.fuse_prepare_row(ctypes.byref(e), None, None, sides, 2, 3) == -1
    # CSR: nnz beyond int32 offsets, nnz > rows * cols
    big = L.CsrDesc(None, None, None, 0, 1 << 20, 1 << 20, 1 << 31)
    assert lib.fuse_prepare_row(ctypes.byref(e), None, ctypes.byref(big), sides, 0, 3) in (-1, -3)
    assert lib.fuse_prepare_outer(ctypes.byref(e), ctypes.byref(L.CsrDesc(None, None, None, 0, 4, 4, 17)),
                                  ctypes.byref(L.Dense(None, 4, 3, 3)), ctypes.byref(L.Dense(None, 4, 3, 3)),
                                  None, 0, 1) == -2
    # the structure check rejects NULL arrays and impossible counts on the host, before any device call
    assert lib.fuse_check_csr(None, None) == -1
    assert lib.fuse_check_csr(ctypes.byref(L.CsrDesc(None, None, None, 0, 4, 4, 3)), None) == -1
    assert b"NULL CSR array" in lib.fuse_last_error()
    assert lib.fuse_check_csr(ctypes.byref(L.CsrDesc(None, None, None, 0, 4, 4, 17)), None) == -2
    # rows * cols beyond int64 must not trip the nnz <= rows * cols test
    huge = L.CsrDesc(None, None, None, 1, 1 << 40, 1 << 30, 1 << 40)
    e3, keep3 = F.api._expr([("main",), ("rowsum",)])
    assert lib.fuse_prepare_row(ctypes.byref(e3), None, ctypes.byref(huge), None, 0, 0) == 0
    # Outer: factor shapes
    ok = L.CsrDesc(None, None, None, 0, 4, 6, 5)
    e2, keep2 = F.api._expr([("main",), ("uvdot",), ("mul",)])
    assert lib.fuse_prepare_outer(ctypes.byref(e2), ctypes.byref(ok), ctypes.byref(L.Dense(None, 4, 3, 3)),
                                  ctypes.byref(L.Dense(None, 6, 3, 3)), None, 0, 1) == 0
    assert lib.fuse_prepare_outer(ctypes.byref(e2), ctypes.byref(ok), ctypes.byref(L.Dense(None, 6, 3, 3)),
                                  ctypes.byref(L.Dense(None, 4, 3, 3)), None, 0, 1) == -2
    assert lib.fuse_prepare_outer(ctypes.byref(e2), ctypes.byref(ok), ctypes.byref(L.Dense(None, 4, 3, 3)),
                                  ctypes.byref(L.Dense(None, 6, 3, 3)), None, 0, 2) == -7    # Outer has no row_agg
    for mm in (5, 6):                                                                      # right_mm, left_mm
        assert lib.fuse_prepare_outer(ctypes.byref(e2), ctypes.byref(ok), ctypes.byref(L.Dense(None, 4, 3, 3)),
                                      ctypes.byref(L.Dense(None, 6, 3, 3)), None, 0, mm) == 0


def test_sparse_side_inputs_host_checks(F):
    """FUSE_SIDE_SPARSE: compiles for the calls over a CSR main input, is refused elsewhere, and its descriptor is
    checked on the host (no GPU needed)."""
    from paper_1801_00829_amd import _lib as L
    lib = L.load()
    hdr = open(os.path.join(ROOT, "include", "fuse.h")).read()
    assert re.search(r"FUSE_SIDE_SPARSE\s*=\s*6", hdr) and F.api.SIDE["sparse"] == 6
    shape, nnz = (300, 200), 6000
    sp = (0, None, 5000, shape)
    # sum(X * Y * Z), X, Y, Z sparse: Cell, MAgg and Row over a CSR main input
    F.prepare_cell_csr(XYZ, shape, nnz, [("sparse", sp), ("sparse", (1, None, 7000, shape))], "full")
    src = F.last_source()
    assert "fuse_side_kind[] = {6, 6, -1}" in src and "fuse_side_rp64[] = {false, true, false}" in src
    F.prepare_magg_csr([XYZ[:3], [("main",), ("side", 1), ("mul",)]], shape, nnz, [("sparse", sp), ("sparse", sp)])
    F.prepare_row([("main",), ("side", 0), ("mul",), ("rowsum",), ("main",), ("mul",)], shape, [("sparse", sp)], "col_t",
                  nnz=nnz)
    # 32- and 64-bit offsets of the side are different kernels
    k32 = (F.prepare_cell_csr(XYZ[:3], shape, nnz, [("sparse", sp)], "full"), F.last_kernel())[1]
    k64 = (F.prepare_cell_csr(XYZ[:3], shape, nnz, [("sparse", (1, None, 5000, shape))], "full"), F.last_kernel())[1]
    assert k32 != k64
    # refused: dense main inputs, Outer, bodies with k-vectors
    for call in (lambda: F.prepare_cell(XYZ, shape, [("sparse", sp), ("sparse", sp)], "full"),
                 lambda: F.prepare_magg([XYZ], shape, [("sparse", sp), ("sparse", sp)]),
                 lambda: F.prepare_row(XYZ, shape, [("sparse", sp), ("sparse", sp)], "full"),
                 lambda: F.prepare_outer([("main",), ("uvdot",), ("mul",), ("side", 0), ("mul",)], shape, 4, nnz,
                                         [("sparse", sp)], "full"),
                 lambda: F.prepare_row([("main",), ("side", 1), ("mul",), ("main",), ("side", 0), ("matmult",), ("outerk",)],
                                       shape, [("rhs", (shape[1], 3)), ("sparse", sp)], "col_t", nnz=nnz)):
        with pytest.raises(F.FuseError) as e:
            call()
        assert e.value.code == -7, str(e.value)
    # the descriptor: NULL, wrong shape, too many cells for 32-bit offsets
    e_, keep = F.api._expr(XYZ[:3])
    xs = L.CsrDesc(None, None, None, 0, shape[0], shape[1], nnz)
    sides = (L.Side * 1)()
    sides[0].kind = 6
    assert lib.fuse_prepare_cell_csr(ctypes.byref(e_), ctypes.byref(xs), sides, 1, 1) == -1
    assert b"sp is NULL" in lib.fuse_last_error()
    bad = L.CsrDesc(None, None, None, 0, shape[0], shape[1] + 1, 10)
    sides[0].sp = ctypes.pointer(bad)
    assert lib.fuse_prepare_cell_csr(ctypes.byref(e_), ctypes.byref(xs), sides, 1, 1) == -2
    bad = L.CsrDesc(None, None, None, 0, shape[0], shape[1], 1 << 31)
    sides[0].sp = ctypes.pointer(bad)
    assert lib.fuse_prepare_cell_csr(ctypes.byref(e_), ctypes.byref(xs), sides, 1, 1) == -1
    # a launching call wants the side's arrays
    good = L.CsrDesc(None, None, None, 0, shape[0], shape[1], 10)
    sides[0].sp = ctypes.pointer(good)
    assert lib.fuse_prepare_cell_csr(ctypes.byref(e_), ctypes.byref(xs), sides, 1, 1) == 0


def test_row_type_checking_and_sparse_safety(F):
    dot_v = [("main",), ("side", 0), ("dot",)]
    F.prepare_row(dot_v, (100, 10), [("rowvec", None)], "none")            # scalar result, per row
    F.prepare_row(dot_v, (100, 10), [("rowvec", None)], "full")
    with pytest.raises(F.FuseError) as e:
        F.prepare_row(dot_v, (100, 10), [("rowvec", None)], "col")          # column sums of a scalar
    assert e.value.code == -3
    with pytest.raises(F.FuseError) as e:
        F.prepare_row([("side", 0), ("rowsum",)], (100, 10), [("colvec", None)], "none")   # rowsum of a scalar
    assert e.value.code == -3
    # two reduction stages: rowsum(X * rowsum(X))
    nested = [("main",), ("main",), ("rowsum",), ("mul",), ("rowsum",)]
    F.prepare_row(nested, (100, 10), [], "none")
    src = F.last_source()
    assert "#define FUSE_NSTAGE 2" in src and re.search(r"const double (v\d+_0) = a \* red\[0\];\s+part\[1\] \+= \1;", src)
    # CSR: sparse-safe bodies compile, others are rejected with FUSE_EDESC
    F.prepare_row([("main",), ("side", 0), ("mul",), ("abs",)], (100, 10), [("matrix", None)], "col", nnz=50)
    for bad in ([("main",), ("const", 1.0), ("add",)], [("main",), ("exp",)],
                [("side", 0), ("rowsum",), ("main",), ("mul",)], [("main",), ("side", 0), ("add",), ("rowsum",)]):
        with pytest.raises(F.FuseError) as e:
            F.prepare_row(bad, (100, 10), [("matrix", None)], "col", nnz=50)
        assert e.value.code == -3 and "sparse-safe" in str(e.value)
    # dense Row limit on the width of reductions
    with pytest.raises(F.FuseError) as e:
        F.prepare_row(dot_v, (10, 40000), [("rowvec", None)], "none")
    assert e.value.code == -7
    F.prepare_row(dot_v, (10, 5000), [("rowvec", None)], "none")           # several waves per row
    assert "#define FUSE_WPR 4" in F.last_source()


def test_row_out_count_follows_result_kind_and_variant(F):
    """fuse_row_out_count: the library, not the binding, derives the size of a Row result from the kind of the
    body's result (row vector, per-row scalar, k-vector, row (x) k-vector) and the variant of Table 1."""
    from paper_1801_00829_amd import _lib as L, api
    lib = L.load()

    def count(expr, shape, sides, agg, nnz=None):
        e, keep = api._expr(expr)
        sa, ns = api._sides(sides, shape[0], shape[1])
        c = ctypes.c_int64(-1)
        if nnz is None:
            xd = L.Dense(None, shape[0], shape[1], max(shape[1], 1))
            rc = lib.fuse_row_out_count(ctypes.byref(e), ctypes.byref(xd), None, sa, ns, api.AGG[agg], ctypes.byref(c))
        else:
            xs = L.CsrDesc(None, None, None, 0, shape[0], shape[1], nnz)
            rc = lib.fuse_row_out_count(ctypes.byref(e), None, ctypes.byref(xs), sa, ns, api.AGG[agg], ctypes.byref(c))
        return rc, c.value

    m, n, k = 70, 30, 4
    vec = [("main",), ("side", 0), ("mul",)]                                   # row vector
    sc = [("main",), ("side", 0), ("dot",)]                                    # per-row scalar
    kv = [("main",), ("side", 0), ("matmult",)]                                # k-vector
    vk = [("main",), ("main",), ("side", 0), ("matmult",), ("outerk",)]        # row (x) k-vector
    rv, rhs = [("rowvec", None)], [("rhs", (n, k))]
    assert count(vec, (m, n), rv, "none") == (0, m * n)
    assert count(vec, (m, n), rv, "none", nnz=123) == (0, 123)                 # on the pattern of a CSR input
    assert count(vec, (m, n), rv, "row") == (0, m)
    assert count(vec, (m, n), rv, "col") == (0, n) and count(vec, (m, n), rv, "col_t") == (0, n)
    assert count(vec, (m, n), rv, "full") == (0, 1)
    assert count(sc, (m, n), rv, "none") == (0, m) and count(sc, (m, n), rv, "full") == (0, 1)
    assert count(kv, (m, n), rhs, "none") == (0, m * k) and count(kv, (m, n), rhs, "col") == (0, k)
    assert count(kv, (m, n), rhs, "full") == (0, 1)
    assert count(vk, (m, n), rhs, "col_t") == (0, n * k)
    # variants a result kind does not have, and a NULL result pointer: errors, the count is left alone
    assert count(sc, (m, n), rv, "row") == (-3, -1)
    assert count(kv, (m, n), rhs, "row") == (-3, -1)
    assert count(vk, (m, n), rhs, "none") == (-3, -1)
    e, keep = api._expr(vec)
    xd = L.Dense(None, m, n, n)
    sa, ns = api._sides(rv, m, n)
    assert lib.fuse_row_out_count(ctypes.byref(e), ctypes.byref(xd), None, sa, ns, api.AGG["row"], None) == -1


def test_row_matrix_rhs_type_checking(F):
    """vectMatMult / vectOuterMultAdd bodies (Sec. 4.2 Row template; Fig. 8g): kinds, shapes, limits."""
    xv = [("main",), ("side", 0), ("matmult",)]                           # X V  -> one k-vector per row
    F.prepare_row(xv, (1000, 100), [("rhs", (100, 4))], "none")            # m x k output
    assert "#define FUSE_KDIM 4" in F.last_source()
    F.prepare_row(xv, (1000, 100), [("rhs", (100, 4))], "col")             # k column sums
    txxv = [("main",)] + xv + [("outerk",)]                               # t(X) (X V): n x k
    F.prepare_row(txxv, (1000, 100), [("rhs", (100, 4))], "col_t")
    # equal sub-expressions are emitted once: Q = P * (X V) is used twice in the MLogreg core
    q = xv + [("side", 1), ("mul",)]
    core = [("main",)] + q + q + [("rowsum",), ("side", 1), ("mul",), ("sub",), ("outerk",)]
    F.prepare_row(core, (1000, 100), [("rhs", (100, 4)), ("kvec", (1000, 4))], "col_t")
    assert "#define FUSE_NRED 4" in F.last_source()                       # one X V product, not two
    bad = [
        (xv, [("rhs", (99, 4))], "none", -2),                            # V needs n rows
        (xv, [("rhs", (100, 17))], "none", -3),                           # k beyond FUSE_MAX_K
        (xv + [("side", 1), ("mul",)], [("rhs", (100, 4)), ("kvec", (1000, 3))], "none", -3),   # k mismatch
        (xv + [("side", 1), ("mul",)], [("rhs", (100, 4)), ("kvec", (999, 4))], "none", -2),    # kvec rows
        (txxv, [("rhs", (100, 4))], "none", -3),                          # n x k values only as column aggregate
        ([("main",), ("side", 0), ("outerk",)], [("rowvec", None)], "col_t", -3),   # outerk needs a k-vector
        ([("side", 0), ("main",), ("matmult",)], [("rhs", (100, 4))], "none", -3),  # operand order
        (xv, [("rhs", (100, 4))], "row", -3),                             # rowSums of a k-vector: use ROWSUM
    ]
    for expr, sides, agg, code in bad:
        with pytest.raises(F.FuseError) as e:
            F.prepare_row(expr, (1000, 100), sides, agg)
        assert e.value.code == code, (expr, sides, agg, e.value.code, str(e.value))
    F.prepare_row(txxv, (100, 2000), [("rhs", (2000, 4))], "col_t")         # several waves per row
    assert "#define FUSE_WPR 4" in F.last_source()
    F.prepare_row(txxv, (100, 784), [("rhs", (784, 10))], "col_t")           # the MLogreg shape of Mnist
    assert "#define FUSE_KDIM 10" in F.last_source()
    F.prepare_row(txxv, (100, 1000), [("rhs", (1000, 8))], "col_t")          # same launch shape, other k: its own plan
    assert "#define FUSE_KDIM 8" in F.last_source()
    with pytest.raises(F.FuseError) as e:                                 # register budget: ceil(n/2048)*2*k <= 48
        F.prepare_row(txxv, (100, 6000), [("rhs", (6000, 16))], "col_t")
    assert e.value.code == -7
    # CSR main input: the products run over the stored cells of a row; the row-vector operand must be sparse-safe
    F.prepare_row(xv, (1000, 100), [("rhs", (100, 4))], "none", nnz=500)
    F.prepare_row(txxv, (1000, 100), [("rhs", (100, 4))], "col_t", nnz=500)
    assert "#define FUSE_RESULT_KIND 4" in F.last_source() and "fuse_csr_rhs" in F.last_source()
    F.prepare_row(core, (1000, 100), [("rhs", (100, 4)), ("kvec", (1000, 4))], "col_t", nnz=500)
    for bad in ([("side", 1), ("side", 0), ("matmult",)],                                   # dense row vector times V
                [("main",), ("const", 1.0), ("add",), ("side", 0), ("matmult",)],           # (X + 1) V
                [("side", 1), ("main",), ("side", 0), ("matmult",), ("outerk",)]):          # t(dense) (X V)
        with pytest.raises(F.FuseError) as e:
            F.prepare_row(bad, (1000, 100), [("rhs", (100, 4)), ("rowvec", None)], "col_t", nnz=500)
        assert e.value.code == -3 and "sparse-safe" in str(e.value)


def test_every_operator_compiles(F):
    un = ["neg", "abs", "sqrt", "exp", "log", "pow2", "sign", "neq0", "sigmoid"]
    bi = ["add", "sub", "mul", "div", "min", "max", "pow", "lt", "le", "gt", "ge", "eq", "ne"]
    expr = [("main",)]
    for u in un:
        expr += [(u,)]
    for b in bi:
        expr += [("side", 0), (b,)]
    F.prepare_cell(expr, (16, 16), [("matrix", None)], "full")
    F.prepare_cell(expr, (16, 16), [("colvec", None)], "row")              # 2-D form of the Cell skeleton
    assert F.last_kernel().startswith("fuse_cell2d_")
    F.prepare_outer(expr + [("uvdot",), ("mul",)], (16, 16), 5, 20, [("rowvec", None)], "none")


def test_binding_rejects_host_tensors(F):
    """A host tensor's pointer would be dereferenced on the device (a GPU fault, not an error): the binding
    refuses it before calling the library."""
    import torch
    x = torch.ones(4, 4, dtype=torch.float64)
    empty_csr = F.Csr(torch.zeros(5, dtype=torch.int32), torch.zeros(0, dtype=torch.int32),
                      torch.zeros(0, dtype=torch.float64), (4, 4))
    for call in (lambda: F.fuse_cell([("main",)], x, [], "full"),
                 lambda: F.fuse_magg([[("main",)]], x, []),
                 lambda: F.fuse_row([("main",), ("rowsum",)], x, [], "none"),
                 lambda: F.fuse_row([("main",)], empty_csr, [], "full"),
                 lambda: F.fuse_outer([("uvdot",)], empty_csr, x, x, [], "full"),
                 lambda: F.check_csr(empty_csr)):
        with pytest.raises(ValueError, match="CUDA"):
            call()


def test_descriptor_length_limits(F):
    """A body may have up to 4096 tokens: the longest one parses and compiles (hipRTC, no device), one
    token more is rejected; so is an empty body."""
    body = [("main",)]
    for i in range(2047):
        body += [("const", 1.0 + 1.0 / (i + 2)), ("mul",)]
    assert len(body) == 4095
    body += [("abs",)]
    assert len(body) == 4096
    F.prepare_cell(body, (16, 16), [], "full")
    with pytest.raises(F.FuseError) as e:
        F.prepare_cell(body + [("neg",)], (16, 16), [], "full")
    assert e.value.code == -1
    with pytest.raises(F.FuseError):
        F.prepare_cell([], (16, 16), [], "full")


def test_plan_cache_is_thread_safe(F):
    """Several host threads prepare the same and different operators at once: every call succeeds and equal
    requests end up on one plan (threads that meet on a new plan may each compile it; one copy is kept)."""
    import threading
    F.cache_clear()
    bodies = [[("main",), ("const", float(c)), ("mul",), ("side", 0), ("add",)] for c in range(3, 7)]
    errors, names = [], {}

    def work(tid):
        try:
            for rep in range(3):
                for j, body in enumerate(bodies):
                    F.prepare_cell(body, (64, 32), [("matrix", None)], "full")
                    names.setdefault(j, set()).add(F.last_kernel())
                    F.prepare_row([("main",), ("side", 0), ("dot",), ("main",), ("mul",)], (50, 20), [("rowvec", None)],
                                  "col_t")
        except Exception as e:            # noqa: BLE001 - reported below
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert all(len(v) == 1 for v in names.values()), names          # one kernel name per body
    assert len({next(iter(v)) for v in names.values()}) == len(bodies)
    hits, misses, _ = F.cache_stats()
    assert hits + misses == 6 * 3 * len(bodies) * 2
    assert len(bodies) + 1 <= misses <= 6 * (len(bodies) + 1)


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    from paper_1801_00829_amd import _lib as L
    monkeypatch.setattr(L, "_lib", None)
    monkeypatch.setattr(L, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        L.load()


def test_cost_arithmetic_matches_the_papers_worked_example():
    """bytes / bandwidth helper of the benchmark against the example printed with the cost model."""
    import importlib
    bench = importlib.import_module("bench")
    vals = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "cost_model_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    nbytes = vals["rows"] * vals["cols"] * vals["bytes_per_cell"]
    assert bench.seconds_at(nbytes, vals["bandwidth_GBps"]) == vals["seconds"]
    assert bench.gbps(nbytes, vals["seconds"]) == vals["bandwidth_GBps"]


def test_code_objects_persist_in_the_cache_directory(F, tmp_path, monkeypatch):
    """FUSE_CACHE_DIR: a compiled body is written there and a later plan-cache miss (here: after clearing
    the in-memory cache) takes it from there without compiling; a damaged file is ignored and rewritten."""
    monkeypatch.setenv("FUSE_CACHE_DIR", str(tmp_path))
    body = [("main",), ("const", 0.123456789), ("mul",), ("abs",), ("sqrt",)]
    F.cache_clear()
    F.prepare_cell(body, (64, 64), [], "full")
    files = sorted(os.listdir(tmp_path))
    assert len(files) == 1 and files[0].startswith(F.last_kernel() + "-") and files[0].endswith(".co")
    hits, misses, ms = F.cache_stats()
    assert (hits, misses) == (0, 1) and ms > 0 and F.cache_disk_hits() == 0
    blob = open(os.path.join(tmp_path, files[0]), "rb").read()
    assert blob[:8] == b"FUSECO01" and len(blob) > 1000
    # a fresh in-memory cache: the miss is served from the directory
    F.cache_clear()
    F.prepare_cell(body, (64, 64), [], "full")
    hits, misses, ms = F.cache_stats()
    assert (hits, misses) == (0, 1) and ms == 0.0 and F.cache_disk_hits() == 1
    # another body is another file
    F.prepare_cell(body + [("neg",)], (64, 64), [], "full")
    assert len(os.listdir(tmp_path)) == 2 and F.cache_disk_hits() == 1
    # a truncated and a bit-flipped file are ignored, recompiled and rewritten whole
    for damage in (lambda b: b[:len(b) // 2], lambda b: b[:200] + bytes([b[200] ^ 1]) + b[201:]):
        open(os.path.join(tmp_path, files[0]), "wb").write(damage(blob))
        F.cache_clear()
        F.prepare_cell(body, (64, 64), [], "full")
        assert F.cache_disk_hits() == 0 and F.cache_stats()[2] > 0
        assert open(os.path.join(tmp_path, files[0]), "rb").read() == blob
    # a directory that cannot be written is not an error
    monkeypatch.setenv("FUSE_CACHE_DIR", str(tmp_path / "missing" / "dir"))
    F.cache_clear()
    F.prepare_cell(body, (64, 64), [], "full")
    assert F.cache_disk_hits() == 0
    F.cache_clear()
