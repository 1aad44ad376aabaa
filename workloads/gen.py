"""Seeded random input generators (numpy PCG64).  No arithmetic of the method here.

The paper's micro-benchmarks use synthetic matrices made with ``rand``
(Sec. 5.1 "Datasets"; shapes and sparsities in Sec. 5.2); these generators
stand in for that with fixed seeds.
"""
import numpy as np

BASE_SEED = 180100829


def seed_for(config: int, tensor: int) -> int:
    """Seed of tensor number ``tensor`` of workload number ``config``."""
    return BASE_SEED + 100 * int(config) + int(tensor)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(int(seed)))


def dense_uniform(m, n, lo, hi, seed):
    """m x n float64, entries uniform in [lo, hi)."""
    a = _rng(seed).random((int(m), int(n)))
    if lo != 0.0 or hi != 1.0:
        a *= (hi - lo)
        a += lo
    return a


def dense_normal(m, n, seed):
    """m x n float64, entries standard normal."""
    return _rng(seed).standard_normal((int(m), int(n)))


def _positive_uniform(rng, k):
    """k values uniform in (0, 1): a drawn 0.0 is redrawn, so no stored zeros."""
    v = rng.random(int(k))
    bad = np.flatnonzero(v == 0.0)
    while bad.size:
        v[bad] = rng.random(bad.size)
        bad = bad[v[bad] == 0.0]
    return v


def _bernoulli_block(args):
    """Stored cells of rows [r0, r1) of an m x n Bernoulli(density) pattern."""
    seed, b, r0, r1, n, density = args
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(b)])))
    total = (r1 - r0) * n
    if density >= 1.0:
        flat = np.arange(total, dtype=np.int64)
    else:
        parts, pos = [], -1
        while total > 0 and density > 0.0:
            gaps = rng.geometric(density, size=int(total * density * 1.05) + 1024)
            flat = pos + np.cumsum(gaps, dtype=np.int64)
            keep = flat < total
            parts.append(flat[keep])
            if not keep.all():
                break
            pos = int(flat[-1])
        flat = np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)
    rows = flat // n
    cols = (flat - rows * n).astype(np.int32)
    counts = np.bincount(rows, minlength=r1 - r0).astype(np.int64)
    return counts, cols, _positive_uniform(rng, cols.size)


def csr_bernoulli(m, n, density, seed, rows_per_block=1 << 16, workers=None):
    """CSR pattern with independent Bernoulli(density) cells.

    Rows are drawn in fixed blocks of ``rows_per_block`` rows, block b from its
    own stream seeded by (seed, b), so the result does not depend on how many
    worker threads draw the blocks.  Within a block the stored positions are
    geometric gaps along the row-major cell order, which is exactly an i.i.d.
    Bernoulli process over the cells: per-row counts are Binomial(n, density),
    columns within a row are distinct and ascending.  Values are uniform in (0, 1).
    Returns (rowptr int64[m+1], colidx int32[nnz], vals float64[nnz]).
    """
    m, n = int(m), int(n)
    tasks = [(seed, b, r0, min(r0 + rows_per_block, m), n, float(density))
             for b, r0 in enumerate(range(0, m, rows_per_block))]
    if len(tasks) > 1:
        import os
        from concurrent.futures import ThreadPoolExecutor
        nw = workers or min(16, os.cpu_count() or 1)
        with ThreadPoolExecutor(max_workers=nw) as ex:
            res = list(ex.map(_bernoulli_block, tasks))
    else:
        res = [_bernoulli_block(t) for t in tasks]
    rowptr = np.zeros(m + 1, dtype=np.int64)
    if res:
        np.cumsum(np.concatenate([r[0] for r in res]), out=rowptr[1:])
        colidx = np.concatenate([r[1] for r in res])
        vals = np.concatenate([r[2] for r in res])
    else:
        colidx, vals = np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float64)
    return rowptr, colidx, vals


def csr_fixed_per_row(m, n, k, seed):
    """CSR with exactly k stored cells in every row, columns uniform without
    replacement and ascending; values uniform in (0, 1)."""
    m, n, k = int(m), int(n), int(k)
    assert 0 <= k <= n
    rng = _rng(seed)
    # argsort of random keys gives a uniform random k-subset per row
    keys = rng.random((m, n))
    colidx = np.sort(np.argsort(keys, axis=1)[:, :k], axis=1).astype(np.int32).reshape(-1)
    rowptr = np.arange(m + 1, dtype=np.int64) * k
    return rowptr, colidx, _positive_uniform(rng, colidx.size)


def csr_skewed(m, n, density, n_long, long_fraction, seed):
    """Bernoulli(density) pattern in which ``n_long`` randomly chosen rows are
    refilled at density ``long_fraction`` (a few very long rows among short
    ones) -- a stress input for nnz-balanced row assignment."""
    m, n = int(m), int(n)
    rng = _rng(seed)
    rowptr, colidx, vals = csr_bernoulli(m, n, density, seed + 7)
    long_rows = set(rng.choice(m, size=min(int(n_long), m), replace=False).tolist()) if m else set()
    parts_c, parts_v, counts = [], [], np.zeros(m, dtype=np.int64)
    for i in range(m):
        if i in long_rows:
            c = np.flatnonzero(rng.random(n) < long_fraction).astype(np.int32)
            v = _positive_uniform(rng, c.size)
        else:
            c = colidx[rowptr[i]:rowptr[i + 1]]
            v = vals[rowptr[i]:rowptr[i + 1]]
        parts_c.append(c)
        parts_v.append(v)
        counts[i] = c.size
    rp = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(counts, out=rp[1:])
    cc = np.concatenate(parts_c) if parts_c else np.zeros(0, dtype=np.int32)
    vv = np.concatenate(parts_v) if parts_v else np.zeros(0, dtype=np.float64)
    return rp, cc.astype(np.int32), vv
