"""Benchmark of the fused-operator hot path on one MI355X.

A step is one pass of the whole hot path: the five fused operators (Cell, MAgg,
Row dense, Row CSR, Outer) on the benchmark workloads, inputs resident in HBM.
Prints ONE JSON line: whole-step effective GB/s (algorithmic bytes of the five
operators / step time), a per-template breakdown, the roofline of the dominant
kernel, and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--templates cell,magg,...] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak
ALL = ("cell", "magg", "row_dense", "row_csr", "outer")

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE at the full
# workload sizes in this launch configuration, scaled by what the same counters read for
# the 1 GiB copy probe (x2.000 for FETCH_SIZE, x1.000 for WRITE_SIZE); the summary is
# profiles/bench_all_templates_hbm_traffic.txt.  Reported as roofline.traffic.
MEASURED_TRAFFIC_BYTES = {"cell": 24.07e6, "magg": 2400.13e6, "row_dense": 808.90e6,
                          "row_csr": 1379.26e6, "outer": 4840.86e6}


def seconds_at(nbytes, gbps_):
    """Time to move nbytes at gbps_ GB/s (1 GB = 1e9 bytes)."""
    return nbytes / (gbps_ * 1e9)


def gbps(nbytes, seconds):
    return nbytes / seconds / 1e9


def _cpu_baseline(names, host):
    """The CPU oracle, as it stands, on the host copies of the same workloads (full size)."""
    from oracle import ops, plans
    total_bytes, total_s, parts, results = 0, 0.0, [], {}
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
        dt = time.perf_counter() - t0
        total_bytes += w["bytes"]
        total_s += dt
        parts.append("%s %.2f s" % (name, dt))
        results[name] = r
    base = {"value": round(gbps(total_bytes, total_s), 3), "unit": "GB/s", "cores": ops.threads(),
            "kind": "oracle", "seconds": round(total_s, 3),
            "sample": "the full workloads, one pass of the unfused operator-at-a-time plans (" +
                      "; ".join(parts) + ")"}
    return base, results


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
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the fused operators are single-device kernels); "
                 "--gpus %d is not supported" % args.gpus)
    names = [n for n in args.templates.split(",") if n]
    for n in names:
        if n not in ALL:
            sys.exit("unknown template %r" % n)

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
        info[name] = {"bytes": int(w["bytes"]), "nnz": int(w.get("nnz", 0))}
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
            info[name]["bytes_compulsory"] = int(w["bytes_compulsory"])
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

    # ---- timed region: exactly K steps; HIP events on the launch stream around every operator
    K = args.steps
    ev = {n: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
          for n in names}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        for name in names:
            a, b = ev[name][k]
            a.record()
            calls[name]()
            b.record()
    torch.cuda.synchronize()
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

    templates = {}
    for name in names:
        ts = sorted(a.elapsed_time(b) for a, b in ev[name])           # milliseconds
        avg = sum(ts) / len(ts)
        e = {"kernel": kernels[name], "bytes": info[name]["bytes"], "avg_us": round(avg * 1e3, 2),
             "min_us": round(ts[0] * 1e3, 2), "median_us": round(ts[len(ts) // 2] * 1e3, 2),
             "GBps": round(gbps(info[name]["bytes"], avg * 1e-3), 1)}
        e["frac_of_hbm_peak"] = round(e["GBps"] / HBM_PEAK_GBPS, 4)
        e["traffic"] = MEASURED_TRAFFIC_BYTES.get(name)
        if info[name]["nnz"]:
            e["nnz_per_s"] = round(info[name]["nnz"] / (avg * 1e-3), 1)
        if "bytes_compulsory" in info[name]:
            e["GBps_compulsory_model"] = round(gbps(info[name]["bytes_compulsory"], avg * 1e-3), 1)
        if name == "cell" and cell_floor is not None:
            e["plain_read_floor"] = cell_floor
        templates[name] = e
    total_bytes = sum(info[n]["bytes"] for n in names)
    dominant = max(names, key=lambda n: templates[n]["avg_us"])
    d = templates[dominant]
    result = {
        "metric": "effective HBM GB/s of one pass over the fused templates (algorithmic bytes / step time)",
        "value": round(gbps(total_bytes, elapsed / K), 1), "unit": "GB/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "one launch each of: " + ", ".join(
            {"cell": "Cell sum(X*Y*Z) 1000x1000", "magg": "MAgg [sum(X*Y),sum(X*Z),sum(X^2)] 100000x1000",
             "row_dense": "Row t(X)%*%(w*(X%*%v)) 1e6x100", "row_csr": "Row-CSR t(X)%*%(X%*%v) 1e7x1000 d=0.01",
             "outer": "Outer sum(X*log(U%*%t(V)+1e-15)) 1e5x1e5 d=0.001 r=100"}[n] for n in names),
            "seed": W.BASE_SEED},
        "roofline": {"bound": "hbm", "kernel": d["kernel"], "template": dominant, "achieved": d["GBps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(d["GBps"] / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(dominant),
                     "traffic_GBps": round(gbps(MEASURED_TRAFFIC_BYTES.get(dominant), d["avg_us"] * 1e-6), 1),
                     "note": ("Outer: algorithmic bytes by the gather model (one V row per non-zero); frac > 1 means "
                              "gathers served by L2 (column panels), see traffic") if dominant == "outer" else ""},
        "templates": templates,
        "plan_cache": {"hits": hits, "misses": misses, "compile_ms": round(compile_ms, 1)},
        "hip_graph_replay": graph,
    }
    if not args.no_cpu_baseline:
        base, refs = _cpu_baseline(names, host)
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
