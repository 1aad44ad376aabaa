"""Maximum sizes: a CSR matrix with more than 2^31 stored cells (int64 row offsets), built on the
device, through the CSR Row skeletons, the sparse Cell form and the Outer template.  The oracle
cannot hold this matrix in seconds, so the checks are closed forms that are exact in fp64:
every row stores the same number of ones at columns base + 5 t, base = row % 5."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

PER_ROW = 600
ROWS = 3_600_000            # 2.16e9 stored cells > 2^31
COLS = 5 * PER_ROW


def _build():
    import torch
    import paper_1801_00829_amd as F
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2**30:
        pytest.skip("needs 60 GiB of free device memory")
    nnz = ROWS * PER_ROW
    assert nnz > 2**31
    rowptr = torch.arange(ROWS + 1, dtype=torch.int64, device="cuda") * PER_ROW
    colidx = torch.empty(nnz, dtype=torch.int32, device="cuda")
    chunk = 30_000 * PER_ROW                      # whole rows per chunk
    t = (torch.arange(PER_ROW, dtype=torch.int32, device="cuda") * 5).repeat(30_000)
    for p0 in range(0, nnz, chunk):
        r0 = p0 // PER_ROW
        rows = min(30_000, ROWS - r0)
        base = (torch.arange(r0, r0 + rows, dtype=torch.int64, device="cuda") % 5).to(torch.int32)
        colidx[p0:p0 + rows * PER_ROW] = t[:rows * PER_ROW] + base.repeat_interleave(PER_ROW)
    vals = torch.ones(nnz, dtype=torch.float64, device="cuda")
    return F.Csr(rowptr, colidx, vals, (ROWS, COLS)), nnz


@pytest.fixture(scope="module")
def big():
    import torch
    x, nnz = _build()
    yield x, nnz
    del x
    torch.cuda.empty_cache()


def test_structure_check_passes(big):
    import paper_1801_00829_amd as F
    F.check_csr(big[0])


@pytest.mark.parametrize("form", ["groups", "stream"])
def test_row_csr_beyond_2_31_cells(big, form, monkeypatch):
    import torch
    import paper_1801_00829_amd as F
    x, nnz = big
    monkeypatch.setenv("FUSE_CSR_STREAM", "1" if form == "stream" else "0")
    per_col = np.array([len(range(c % 5, ROWS, 5)) for c in range(COLS)], dtype=np.float64)
    # t(X) %*% (X %*% v) with v = 1: every row sum is PER_ROW, every column c receives PER_ROW per stored cell
    v = torch.ones(COLS, dtype=torch.float64, device="cuda")
    got = F.fuse_row([("main",), ("side", 0), ("dot",), ("main",), ("mul",)], x, [("rowvec", v)], "col_t").cpu().numpy()
    assert np.array_equal(got, PER_ROW * per_col)
    # row sums and the full sum of X * colvec with an integer-valued column vector
    cv = (torch.arange(ROWS, dtype=torch.float64, device="cuda") % 7) + 1
    body = [("main",), ("side", 0), ("mul",)]
    rows = F.fuse_row(body, x, [("colvec", cv)], "row")
    assert torch.equal(rows, cv * PER_ROW)
    full = F.fuse_row(body, x, [("colvec", cv)], "full").cpu().numpy()[0]
    assert full == float(cv.sum().item()) * PER_ROW
    # positions of the last cells: no_agg output at p = nnz - 1 and around 2^31
    out = F.fuse_row(body, x, [("colvec", cv)], "none")
    for p in (0, 2**31 - 1, 2**31, 2**31 + 1, nnz - 1):
        assert out[p].item() == cv[p // PER_ROW].item(), p


def test_sparse_cell_and_outer_beyond_2_31_cells(big):
    import torch
    import paper_1801_00829_amd as F
    x, nnz = big
    # flat form of the sparse Cell template: sum(X^2) = number of stored cells
    assert F.fuse_cell_csr([("main",), ("pow2",)], x, [], "full").cpu().numpy()[0] == float(nnz)
    # Outer: U = 1 (rank 4), V_j = (j % 3 + 1) e_0  =>  U_i . V_j = j % 3 + 1 at every stored cell (i, j)
    r = 4
    u = torch.ones(ROWS, r, dtype=torch.float64, device="cuda")
    vv = torch.zeros(COLS, r, dtype=torch.float64, device="cuda")
    vv[:, 0] = (torch.arange(COLS, device="cuda") % 3 + 1).to(torch.float64)
    per_col = np.array([len(range(c % 5, ROWS, 5)) for c in range(COLS)], dtype=np.float64)
    expect = float((per_col * (np.arange(COLS) % 3 + 1)).sum())
    for panels in ("0", "2"):
        import os
        os.environ["FUSE_OUTER_PANELS"] = panels
        try:
            got = F.fuse_outer([("main",), ("uvdot",), ("mul",)], x, u, vv, [], "full").cpu().numpy()[0]
        finally:
            os.environ.pop("FUSE_OUTER_PANELS", None)
        assert got == expect, (panels, got, expect)


def test_dense_beyond_2_31_elements():
    """Dense inputs with more than 2^31 elements: flat Cell / MAgg index arithmetic, the 2-D form and the
    dense Row skeleton; integer-valued inputs, so every expected value is exact."""
    import torch
    import paper_1801_00829_amd as F
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2**30:
        pytest.skip("needs 60 GiB of free device memory")
    m, n = 2_200_000, 1000
    assert m * n > 2**31
    x = torch.ones(m, n, dtype=torch.float64, device="cuda")
    x[-1, -1] = 3.0                                   # the very last element must be seen exactly once
    x[2**31 // n, (2**31) % n] = 5.0                  # and the one at flat index 2^31
    y = torch.full((m, n), 2.0, dtype=torch.float64, device="cuda")
    total = float(m) * n + 2.0 + 4.0
    assert F.fuse_cell([("main",), ("side", 0), ("mul",)], x, [("matrix", y)], "full").cpu().numpy()[0] == 2.0 * total
    got = F.fuse_magg([[("main",), ("side", 0), ("mul",)], [("main",), ("pow2",)]], x, [("matrix", y)]).cpu().numpy()
    assert got[0] == 2.0 * total and got[1] == float(m) * n - 2.0 + 9.0 + 25.0
    # 2-D form: row vector side; column and row aggregates
    rv = (torch.arange(n, dtype=torch.float64, device="cuda") % 4) + 1
    cols = F.fuse_cell([("main",), ("side", 0), ("mul",)], x, [("rowvec", rv)], "col").cpu()
    expect = rv.cpu() * m
    expect[-1] += 2.0 * rv[-1].item()
    expect[(2**31) % n] += 4.0 * rv[(2**31) % n].item()
    assert torch.equal(cols, expect)
    rows = F.fuse_cell([("main",)], x, [], "row")
    assert rows[0].item() == n and rows[-1].item() == n + 2.0 and rows[2**31 // n].item() == n + 4.0
    # dense Row: t(X) %*% (X %*% v) with v = 1
    v = torch.ones(n, dtype=torch.float64, device="cuda")
    out = F.fuse_row([("main",), ("side", 0), ("dot",), ("main",), ("mul",)], x, [("rowvec", v)], "col_t").cpu().numpy()
    # q_i = n except the two marked rows; out[c] = sum_i x_ic q_i
    q_last, q_mid = n + 2.0, n + 4.0
    base = float(m - 2) * n + q_last + q_mid
    exp = np.full(n, base)
    exp[-1] += 2.0 * q_last
    exp[(2**31) % n] += 4.0 * q_mid
    assert np.array_equal(out, exp)
    del x, y
    torch.cuda.empty_cache()


def test_narrow_dense_beyond_2_31_elements():
    """Narrow contiguous matrices with more than 2^31 elements: the dense Row skeleton with its rows staged
    through shared memory (50 columns) and the one-wave-per-tile matrix-unit form of t(X) %*% (X %*% V)
    (100 columns); integer-valued inputs, so every expected value is exact."""
    import torch
    import paper_1801_00829_amd as F
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2**30:
        pytest.skip("needs 40 GiB of free device memory")
    txv = [("main",), ("side", 0), ("dot",), ("main",), ("mul",)]
    txxv = [("main",), ("main",), ("side", 0), ("matmult",), ("outerk",)]
    for (m, n) in ((44_000_000, 50), (22_000_000, 100)):
        assert m * n > 2**31
        print("narrow large", m, n, flush=True)
        x = torch.ones(m, n, dtype=torch.float64, device="cuda")
        r5, c5 = 2**31 // n, (2**31) % n
        x[-1, -1] = 3.0                               # the very last element must be seen exactly once
        x[r5, c5] = 5.0                               # and the one at flat index 2^31
        # t(X) %*% (X %*% v) with v = 1: q_i = n except in the two marked rows
        F.cache_clear()
        v = torch.ones(n, dtype=torch.float64, device="cuda")
        out = F.fuse_row(txv, x, [("rowvec", v)], "col_t").cpu().numpy()
        if n == 50:
            assert "#define FUSE_LDSX 1" in F.last_source()
        q_last, q_mid = n + 2.0, n + 4.0
        exp = np.full(n, float(m - 2) * n + q_last + q_mid)
        exp[-1] += 2.0 * q_last
        exp[c5] += 4.0 * q_mid
        assert np.array_equal(out, exp)
        # t(X) %*% (X %*% V), V[c][j] = c % 3 + j + 1; 4, 8 and 16 classes take the three forms of the products
        for k in (4, 8, 16):
            vk = ((torch.arange(n, device="cuda") % 3)[:, None] + torch.arange(k, device="cuda")[None, :] + 1).to(torch.float64)
            got = F.fuse_row(txxv, x, [("rhs", vk)], "col_t").cpu().numpy().reshape(n, k)
            assert F.last_kernel().startswith("fuse_row_mfma_wave_")
            vh = vk.cpu().numpy()
            s = vh.sum(0)
            qm, ql = s + 4.0 * vh[c5], s + 2.0 * vh[n - 1]
            exp = np.tile((m - 2) * s + qm + ql, (n, 1))
            exp[c5] += 4.0 * qm
            exp[n - 1] += 2.0 * ql
            assert np.array_equal(got, exp), k
            # the same through a body with a per-row k-vector side: W = P * Q with P = 1 in every entry
            pk = torch.ones(m, k, dtype=torch.float64, device="cuda")
            body = [("main",), ("side", 1), ("main",), ("side", 0), ("matmult",), ("mul",), ("outerk",)]
            got = F.fuse_row(body, x, [("rhs", vk), ("kvec", pk)], "col_t").cpu().numpy().reshape(n, k)
            assert np.array_equal(got, exp), ("k-vector side", k)
            del pk
        del x
        torch.cuda.empty_cache()
