"""Helpers for the GPU parity tests: host arrays -> device tensors, calls, comparisons."""
import numpy as np


def to_dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def dev_sides(sides):
    out = []
    for kind, val in sides:
        if kind == "scalar":
            out.append((kind, float(np.asarray(val).reshape(-1)[0])))
        elif kind == "sparse":                     # (rowptr, colidx, vals, shape[, rowptr64]) on the host
            out.append((kind, dev_csr(*val)))
        else:
            out.append((kind, to_dev(np.asarray(val, dtype=np.float64))))
    return out


def dev_csr(rowptr, colidx, vals, shape, rowptr64=False):
    import torch
    import paper_1801_00829_amd as F
    rp = to_dev(rowptr, torch.int64 if rowptr64 else torch.int32)
    return F.Csr(rp, to_dev(colidx, torch.int32), to_dev(vals), tuple(shape))


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def assert_close(got, ref, scale=None, tol=1e-10, what=""):
    """max |got - ref| <= tol * scale, scale = max |ref| unless a condition-aware
    scale (e.g. the same aggregate of absolute values) is given.  NaNs must match."""
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if got.size == 0:
        return
    nan_g, nan_r = np.isnan(got), np.isnan(ref)
    assert (nan_g == nan_r).all(), (what, "NaN pattern differs", int(nan_g.sum()), int(nan_r.sum()))
    inf_r = np.isinf(ref)
    assert (got[inf_r] == ref[inf_r]).all(), (what, "infinities differ")
    ok = ~(nan_r | inf_r)
    if not ok.any():
        return
    s = np.abs(ref[ok]).max() if scale is None else float(np.max(scale))
    s = max(s, 1e-300)
    err = np.abs(got[ok] - ref[ok]).max()
    assert err <= tol * s, (what, "max abs err %.3e > %.1e * scale %.3e" % (err, tol, s))
