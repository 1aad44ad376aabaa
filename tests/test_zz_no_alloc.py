"""The entry point that allocates nothing, fuse_magg_noalloc, against fuse_magg on the same inputs:
two calls in a row through the C ABI, the second on a smaller input, each compared with the existing
entry point's result (same kernels, same launch shape: the same bits) and with the CPU oracle."""
import os

import numpy as np
import pytest

from oracle import plans
from gpu_util import to_dev, dev_sides, host

pytestmark = pytest.mark.gpu

MAGG = [[("main",), ("side", 0), ("mul",)], [("main",), ("side", 1), ("mul",)], [("main",), ("pow2",)]]


def _inputs(m, n, seed):
    rng = np.random.default_rng(seed)
    return [rng.uniform(-1.0, 1.0, size=(m, n)) for _ in range(3)]


def test_noalloc_magg_matches_fuse_magg_on_two_calls_in_a_row():
    import torch
    import paper_1801_00829_amd as F
    big, small = _inputs(3001, 1000, 11), _inputs(257, 1000, 12)      # 24 MB and 2 MB per matrix, ragged tails
    dev = []
    for x, y, z in (big, small):
        dev.append((to_dev(x), dev_sides([("matrix", y), ("matrix", z)])))
    # the existing entry point: reference results, and the plan compiled and loaded on this device
    want = [host(F.fuse_magg(MAGG, x, s)).copy() for x, s in dev]
    out = [torch.full((3,), float("nan"), dtype=torch.float64, device="cuda") for _ in dev]
    torch.cuda.synchronize()
    mem = torch.cuda.memory_allocated()
    for (x, s), o in zip(dev, out):                                    # two calls in a row, the second smaller
        F.fuse_magg_noalloc(MAGG, x, s, o)
    assert torch.cuda.memory_allocated() == mem
    got = [host(o) for o in out]
    for g, w, (x, y, z) in zip(got, want, (big, small)):
        assert np.array_equal(g, w), (g, w)                            # same kernel, same grid, same order of sums
        ref = plans.magg_xy_xz_xx(x, y, z)
        scale = np.array([np.abs(x * y).sum(), np.abs(x * z).sum(), (x * x).sum()])
        assert (np.abs(g - ref) <= 1e-10 * scale).all(), (g, ref)
    # k = 1: the full aggregate of the Cell template, again large then small, interleaved with the 3-sum operator
    cell = [[("main",), ("side", 0), ("mul",), ("side", 1), ("mul",)]]
    wantc = [host(F.fuse_magg(cell, x, s)).copy() for x, s in dev]
    oc = [torch.full((1,), float("nan"), dtype=torch.float64, device="cuda") for _ in dev]
    for rep in range(3):
        for (x, s), o, o3 in zip(dev, oc, out):
            F.fuse_magg_noalloc(cell, x, s, o)
            F.fuse_magg_noalloc(MAGG, x, s, o3)
        for o, w, o3, w3 in zip(oc, wantc, out, want):
            assert np.array_equal(host(o), w) and np.array_equal(host(o3), w3), rep


def test_noalloc_magg_recorded_into_a_hip_graph():
    """What the entry point is for: a caller under stream capture.  Two calls (a large and a small input) are recorded
    into one HIP graph after one eager call each; the graph is replayed three times with the inputs changed in
    between (and eager work on the same operators between the replays), every replay against the eager result."""
    import torch
    import paper_1801_00829_amd as F
    big, small = _inputs(2003, 1000, 21), _inputs(129, 1000, 22)
    dev = [(to_dev(x), dev_sides([("matrix", y), ("matrix", z)])) for x, y, z in (big, small)]
    out = [torch.zeros(3, dtype=torch.float64, device="cuda") for _ in dev]
    gs = torch.cuda.Stream()
    gs.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(gs):
        for (x, s), o in zip(dev, out):
            F.fuse_magg(MAGG, x, s)                                    # compiled and loaded; the per-device set-up done
            F.fuse_magg_noalloc(MAGG, x, s, o)
    gs.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=gs):
        for (x, s), o in zip(dev, out):
            F.fuse_magg_noalloc(MAGG, x, s, o)
    for rep in range(3):
        for (x, s) in dev:                                             # new values in the same buffers
            x.mul_(1.0 + 0.125 * (rep + 1))
            s[0][1].add_(0.25)
        torch.cuda.synchronize()
        for o in out:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = [host(o).copy() for o in out]
        want = [host(F.fuse_magg(MAGG, x, s)).copy() for x, s in dev]  # eager, between the replays
        for a, b in zip(got, want):
            assert np.array_equal(a, b), (rep, a, b)


def test_noalloc_magg_refuses_what_it_cannot_do_without_allocating():
    import torch
    import paper_1801_00829_amd as F
    x, y, z = _inputs(300, 1000, 13)
    dx, s = to_dev(x), dev_sides([("matrix", y), ("matrix", z)])
    o = torch.zeros(1, dtype=torch.float64, device="cuda")
    fresh = [[("main",), ("side", 0), ("sub",), ("abs",), ("side", 1), ("mul",), ("const", 0.8125), ("add",)]]
    with pytest.raises(F.FuseError) as e:                              # never compiled: nothing may be compiled here
        F.fuse_magg_noalloc(fresh, dx, s, o)
    assert e.value.code == -8, e.value
    F.fuse_magg(fresh, dx, s)
    ref = host(F.fuse_magg(fresh, dx, s)).copy()
    assert np.array_equal(host(F.fuse_magg_noalloc(fresh, dx, s, o)), ref)
    # strided input: the 2-D form has a workspace of its own size, not served here
    with pytest.raises(F.FuseError) as e:
        F.fuse_magg_noalloc(fresh, dx[:, :998], [(k, t[:, :998]) for k, t in s], o)
    assert e.value.code == -7 and "contiguous" in str(e.value), e.value
    # a grid that needs more block partials than the fixed array holds is refused before anything is launched
    os.environ["FUSE_CELL_GRID"] = "9000"
    try:
        with pytest.raises(F.FuseError) as e:
            F.fuse_magg_noalloc(fresh, dx, s, o)
        assert e.value.code == -7 and "block partials" in str(e.value), e.value
    finally:
        del os.environ["FUSE_CELL_GRID"]
    assert np.array_equal(host(F.fuse_magg_noalloc(fresh, dx, s, o)), ref)
