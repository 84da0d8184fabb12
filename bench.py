#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4-gcn] [--f-chunk C]

A step is one gnnagg_aggregate call (chunk addressing, gather, reduce, in-place
concat) over the whole synthetic graph, with the CSR, the row plan and the
features already resident in HBM.  The default workload is the dense
232,965-vertex / 114.6 M-edge graph with 602 fp32 features and GCN weights; the
sparse 2.4 M-vertex bf16 workload is measured after it and reported under "also".  The CSR build and the row plan are per-graph
steps; they are timed separately and reported under "setup".  Prints one JSON
line: edge-features/s, the HBM roofline of the aggregation kernel (algorithmic
bytes / HIP-event time, peak 8 TB/s) and the CPU checker timed on the host
cores on a bounded sample of destination rows of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_F64_PEAK_TFLOPS = 78.6

# HBM-side bytes per aggregation call (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc, summed over the call's
# launches - a narrower last slice gets a launch of its own on dense graphs - and scaled on the copy
# probe: see profiles/aggregate_kernel_*.txt), valid for the kernels as committed with those profiles and
# for f_chunk = 0 only.  Set an entry to None when the kernel changes until the counters are taken again.
MEASURED_TRAFFIC = {
    "c4-gcn": 119.643e9,  # profiles/aggregate_kernel_c4_gcn.txt
    "c5-sum": 13.317e9,   # profiles/aggregate_kernel_c5_sum_bf16.txt
    "c4-gat": 14.677e9,   # profiles/gat_aggregate_kernel_c4_gat.txt
    "c4-hid32-gcn": 6.483e9,  # profiles/aggregate_kernel_c4_hidden32_gcn.txt
}

WORKLOADS = {
    # name: (graph key, op, F, feature dtype, self loops + GCN norm)
    "c4-gcn": ("c4", "wsum", 602, "f32", True),
    "c4-mean": ("c4", "mean", 602, "f32", False),
    "c5-sum": ("c5", "sum", 100, "bf16", False),
    "c5-max": ("c5", "max", 100, "bf16", False),
    "c5-sum-f32": ("c5", "sum", 32, "bf16", False),
    "c5-sum-f16": ("c5", "sum", 16, "bf16", False),
    "c2-mean": ("c2", "mean", 500, "f32", False),
    "c1-gcn": ("c1", "wsum", 1433, "f32", True),
    # attention: F = (heads, channels per head); self-loops, no GCN weights
    "c3-gat": ("c2", "gat", (8, 8), "f32", False),
    "c4-gat": ("c4", "gat", (8, 8), "f32", False),
    # the paper's regime: Combination first, so Aggregation runs at the hidden width 8/16/32 (Section III)
    "c4-hid32-gcn": ("c4", "wsum", 32, "f32", True),
    "c4-hid8-gcn": ("c4", "wsum", 8, "f32", True),
    "c6-hid32-gcn": ("c6", "wsum", 32, "f32", True),
    "c6-hid16-gcn": ("c6", "wsum", 16, "f32", True),
    "c6-hid8-gcn": ("c6", "wsum", 8, "f32", True),
    "c6-hid32-mean": ("c6", "mean", 32, "f32", False),
    "c6-gat": ("c6", "gat", (8, 4), "f32", False),
    # Combination (dense layer F -> H on the matrix cores), alone and as one GCN layer with Combination first
    "c4-combine-32": ("c4", "combine", (602, 32), "f32", False),
    "c4-layer-32": ("c4", "layer", (602, 32), "f32", True),
    # the sparse graph at hidden width 16 after Combination: rows of 64 bytes, two per line; "-ranked" stores
    # the hidden rows in popularity order (gnnagg_rank_sources + out_rows of gnnagg_combine)
    "c5-layer-16": ("c5", "layer", (100, 16), "f32", False),
    "c5-layer-16-ranked": ("c5", "layer-ranked", (100, 16), "f32", False),
}


_GRAPHS = {}


def graph_of(W, gkey):
    """The synthetic graph of a workload, generated once per run."""
    if gkey not in _GRAPHS:
        _GRAPHS.clear()  # one graph at a time: the largest holds ~1 GB of host memory
        _GRAPHS[gkey] = W.graph(gkey)
    return _GRAPHS[gkey]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(nnz, N, F, x_bytes, weighted, f_chunk):
    """Bytes the method itself has to move per call: every neighbour-row slice once per edge, the
    index (and weight) of every edge once per chunk pass, every output element once, the row
    pointers once per chunk pass."""
    P = 1 if (f_chunk <= 0 or f_chunk >= F) else -(-F // f_chunk)
    return nnz * F * x_bytes + P * nnz * (4 + (4 if weighted else 0)) + N * F * 4 + P * (N + 1) * 8


def measure_layer(g, W, torch, workload, steps, warmup, copy_gbs):
    """Combination (X W on the matrix cores) alone, or followed by the GCN aggregation at the hidden width."""
    gkey, opname, (F, H), xdt, gcn = WORKLOADS[workload]
    N, src, dst = graph_of(W, gkey)
    X = torch.from_numpy(W.normal_f32((N, F), seed=13)).cuda()
    Wt = torch.from_numpy(W.normal_f32((F, H), seed=16, std=0.05)).cuda()
    hid = torch.empty((N, H), dtype=torch.float32, device="cuda")
    out = torch.empty((N, H), dtype=torch.float32, device="cuda")
    nnz = 0
    ranked = opname == "layer-ranked"
    rank = None
    if ranked:
        opname = "layer"
    if opname == "layer":
        flags = (g.SELF_LOOPS | g.NORM_SYM) if gcn else 0
        d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(),
                                                flags, want_w=gcn)
        plan = g.gnnagg_plan_rows(d_rp)
        nnz = int(d_ci.shape[0])
        if ranked:  # per graph, like the CSR and the plan
            rank, d_ci = g.gnnagg_rank_sources(N, d_ci)
    aop = g.WSUM if gcn else g.SUM

    def step():
        g.gnnagg_combine(X, Wt, None, False, hid, out_rows=rank)
        if opname == "layer":
            g.gnnagg_aggregate(aop, d_rp, d_ci, d_w, hid, out, 0, plan)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    kern_ms = e0.elapsed_time(e1) / steps
    flop = 2.0 * N * F * H
    b_alg = N * F * 4 + F * H * 4 + N * H * 4
    if opname == "layer":
        b_alg += algorithmic_bytes(nnz, N, H, 4, gcn, 0)
    achieved = b_alg / (kern_ms * 1e-3) / 1e9
    log("%s: %.3f ms per step (combination %.1f GFLOP in fp64 MFMA), %.0f GB/s algorithmic" %
        (workload, kern_ms, flop / 1e9, achieved))
    rec = {"metric": "one layer, Combination first" if opname == "layer" else "Combination (dense layer)",
           "value": (float(nnz) * H if opname == "layer" else flop) / (ms_per_step * 1e-3),
           "unit": "edge-features/s at the hidden width" if opname == "layer" else "flop/s",
           "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": workload, "graph": W.GRAPHS[gkey].name, "N": N, "nnz": nnz, "F": F, "H": H},
           "cpu_baseline": None, "setup": {}}
    if opname == "combine":  # the dense contraction: priced against the fp64 matrix-core peak
        tf = flop / (kern_ms * 1e-3) / 1e12
        rec["roofline"] = {"bound": "mfma", "achieved": tf, "peak": MFMA_F64_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": tf / MFMA_F64_PEAK_TFLOPS, "traffic": None, "kernel": "combine_kernel",
                           "kernel_ms": kern_ms, "flop": flop, "algorithmic_bytes": b_alg,
                           "algorithmic_gbs": achieved, "measured_copy_gbs": copy_gbs}
    else:
        rec["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                           "kernel": "combine_kernel + aggregate_kernel", "kernel_ms": kern_ms,
                           "algorithmic_bytes": b_alg, "measured_copy_gbs": copy_gbs}
    return rec


def measure(g, W, torch, workload, f_chunk, steps, warmup, cpu_baseline, cpu_seconds, copy_gbs, pitched=True):
    """One workload: setup (CSR build, row plan), timed aggregation steps, optional CPU-checker leg."""
    gkey, opname, F, xdt, gcn = WORKLOADS[workload]
    if opname in ("combine", "layer", "layer-ranked"):
        return measure_layer(g, W, torch, workload, steps, warmup, copy_gbs)
    gat = opname == "gat"
    heads, C = F if gat else (1, F)
    F = heads * C
    t0 = time.time()
    N, src, dst = graph_of(W, gkey)
    log("graph %s: N=%d directed edges=%d (%.1fs)" % (gkey, N, len(src), time.time() - t0))
    t0 = time.time()
    X = W.normal_bf16((N, F), seed=13) if xdt == "bf16" else (
        W.bernoulli_f32((N, F), 0.013, seed=13) if gkey == "c1" else W.normal_f32((N, F), seed=13))
    log("features [%d,%d] %s (%.1fs)" % (N, F, xdt, time.time() - t0))

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    d_src, d_dst, d_X = dev(src), dev(dst), dev(X)
    flags = (g.SELF_LOOPS | g.NORM_SYM) if gcn else (g.SELF_LOOPS if gat else 0)
    # ---- per-graph setup: CSR build and row plan (timed, not part of a step)
    g.gnnagg_build_csr(N, d_src, d_dst, flags, want_w=gcn)  # warm-up (allocator, code objects)
    torch.cuda.synchronize()
    t0 = time.time()
    d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, d_src, d_dst, flags, want_w=gcn)
    torch.cuda.synchronize()
    t_csr = time.time() - t0
    t0 = time.time()
    plan = g.gnnagg_plan_rows(d_rp)
    torch.cuda.synchronize()
    t_plan = time.time() - t0
    del d_src, d_dst
    nnz = int(d_ci.shape[0])
    log("device CSR build %.1f ms, row plan %.1f ms, nnz=%d" % (t_csr * 1e3, t_plan * 1e3, nnz))

    out = torch.empty((N, F), dtype=torch.float32, device="cuda")
    if pitched and not gat:
        # rows of X and out start on 128-byte lines (the layout the library recommends: gnnagg_row_pitch);
        # the padding columns are never read or written and are not counted in any byte figure
        Xp = g.pitched_empty(N, F, d_X.dtype)
        Xp.copy_(d_X)
        d_X = Xp
        out = g.pitched_empty(N, F, torch.float32)
    if gat:
        a_s, a_d = W.normal_f32((heads, C), seed=14, std=0.1), W.normal_f32((heads, C), seed=15, std=0.1)
        d_as, d_ad = dev(a_s), dev(a_d)
        d_H, out3 = d_X.view(N, heads, C), out.view(N, heads, C)
        ws = torch.empty(g.gnnagg_gat_workspace_bytes(N, heads, C, plan), dtype=torch.uint8, device="cuda")

        def step():
            g.gnnagg_gat_attention(d_rp, d_ci, d_H, d_as, d_ad, 0.2, False, True, max(f_chunk, 0), plan, out=out3,
                                   workspace=ws)
    else:
        op = {"sum": g.SUM, "wsum": g.WSUM, "mean": g.MEAN, "max": g.MAX}[opname]

        def step():
            g.gnnagg_aggregate(op, d_rp, d_ci, d_w, d_X, out, f_chunk, plan)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # whole timed region: wall clock around K steps; per-step kernel time: HIP events on the launch stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = np.array([a.elapsed_time(b) for a, b in ev])
    ms_per_step = wall * 1e3 / steps
    edge_features = float(nnz) * F
    x_bytes = 2 if xdt == "bf16" else 4
    if gat:  # per edge: the row piece, the index, and one score per head unless the kernel recomputes it from the
        # row piece (heads of 4, 8 or 16 channels); per vertex: H once for the scores, out, scores
        per_edge_score = 0 if C in (4, 8, 16) else heads * 4
        b_alg = nnz * (F * 4 + per_edge_score + 4) + 2 * N * F * 4 + 2 * N * heads * 4 * 2 + (N + 1) * 8
    else:
        f_eff = (g.gnnagg_auto_f_chunk(N, F, g.BF16 if xdt == "bf16" else g.F32, int(d_X.stride(0)), plan)
                 if f_chunk == -1 else f_chunk)
        # priced at ONE pass over the edge list (the smaller figure), whatever chunk width runs: the index and
        # weight re-reads of a chunked run are the method's overhead, not work to take credit for
        b_alg = algorithmic_bytes(nnz, N, F, x_bytes, opname == "wsum", 0)
        b_alg_chunked = algorithmic_bytes(nnz, N, F, x_bytes, opname == "wsum", f_eff)
    kern_ms = float(ms.mean())
    achieved = b_alg / (kern_ms * 1e-3) / 1e9
    # every array once: the floor no gather kernel reaches, reported as distance from the ideal
    compulsory = N * F * x_bytes + N * F * 4 + nnz * (8 if opname == "wsum" else 4) + (N + 1) * 8
    if gat:
        compulsory += 2 * N * heads * 4
    traffic = MEASURED_TRAFFIC.get(workload) if (f_chunk == -1 and pitched) else None  # taken in the default set-up
    log("step %.3f ms wall, kernel mean %.3f ms (min %.3f), %.3e edge-features/s, %.0f GB/s algorithmic" %
        (ms_per_step, kern_ms, ms.min(), edge_features / (ms_per_step * 1e-3), achieved))

    # ---- launch-bound workloads: the same step captured in a HIP graph and replayed (the calls only enqueue
    # kernels, so they can be captured); reported beside the eager figure
    graph_ms = None
    if edge_features < 1e9:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        graph_ms = g0.elapsed_time(g1) / steps
        log("captured in a graph and replayed: %.4f ms per step" % graph_ms)

    # ---- CPU checker on the host cores: bounded sample of destination rows, also the parity check
    cpu = None
    parity = None
    if not (not cpu_baseline):
        import oracle
        threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
        t0 = time.time()
        rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=gcn, threads=threads)
        log("checker CSR build %.1fs on %d threads" % (time.time() - t0, threads))
        rop = {"sum": oracle.SUM, "wsum": oracle.WSUM, "mean": oracle.MEAN, "max": oracle.MAX}.get(opname)

        def checker_rows(rr):
            if gat:
                return oracle.gat_attention_rows(rr, rp, ci, X.reshape(N, heads, C), a_s, a_d, 0.2,
                                                 threads=threads).reshape(len(rr), F)
            return oracle.aggregate_rows(rop, rr, rp, ci, w, X, threads=threads)

        rng = np.random.default_rng(0)
        deg = np.diff(rp)
        probe = np.sort(rng.choice(N, size=min(N, 256), replace=False)).astype(np.int64)
        t0 = time.time()
        checker_rows(probe)
        rate = max(float(deg[probe].sum()) * F / max(time.time() - t0, 1e-4), 1.0)
        want = cpu_seconds * rate / F  # edges to cover in about cpu_seconds
        nrows = int(min(N, max(256, want / max(deg.mean(), 1.0))))
        rows = np.sort(rng.choice(N, size=nrows, replace=False)).astype(np.int64)
        t0 = time.time()
        ref = checker_rows(rows)
        dt = time.time() - t0
        ef = float(deg[rows].sum()) * F
        cpu = {"value": ef / dt, "unit": "edge-features/s", "cores": threads, "kind": "oracle",
               "sample": "%d random destination rows of %s (%.3g edge-features, %.1f s)" % (nrows, workload, ef, dt)}
        got = out[torch.from_numpy(rows).cuda()].cpu().numpy()
        tol = 1e-2 if xdt == "bf16" else 1e-5
        if opname == "max":
            parity = bool(np.array_equal(got.view(np.uint32), ref.view(np.uint32)))
        else:
            parity = bool(np.all(np.abs(got.astype(np.float64) - ref) <= 1e-6 + tol * np.abs(ref)))
        log("checker: %.3e edge-features/s on %d threads; parity on the sample: %s" % (cpu["value"], threads, parity))

    rec = {
        "metric": "aggregated edge-features/sec", "value": edge_features / (ms_per_step * 1e-3),
        "unit": "edge-features/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": workload, "graph": W.GRAPHS[gkey].name, "N": N, "nnz": nnz, "F": F, "op": opname,
                   "f_chunk": f_chunk, "f_chunk_used": (F if gat else (f_eff if 0 < f_eff < F else F)), "x_dtype": xdt, "x_row_pitch": int(d_X.stride(0)),
                   "out_row_pitch": int(out.stride(0))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "kernel": "gat_aggregate_kernel (+ score pass)" if gat else "aggregate_kernel",
                     "per": "library call (all its launches of that kernel; kernel_ms is their sum)",
                     "kernel_ms": kern_ms, "kernel_ms_median": float(np.median(ms)), "kernel_ms_min": float(ms.min()),
                     "algorithmic_bytes": b_alg,
                     "algorithmic_bytes_with_edge_list_rereads": None if gat else b_alg_chunked,
                     "hbm_gbs": (traffic / (kern_ms * 1e-3) / 1e9) if traffic else None,
                     "compulsory_bytes": compulsory,
                     "compulsory_frac": compulsory / (HBM_PEAK_GBS * 1e9) / (kern_ms * 1e-3),
                     "measured_copy_gbs": copy_gbs},
        "cpu_baseline": cpu,
        "parity_on_sample": parity,
        "graph_replay_ms_per_step": graph_ms,
        "setup": {"csr_build_ms": t_csr * 1e3, "row_plan_ms": t_plan * 1e3},
    }
    return rec




def cpu_chunk_sweep(W, workload, widths):
    """The CPU checker in the chunk-outer order of Algorithm 1 over a sweep of chunk widths, whole graph:
    context for the paper's own (CPU) effect, not a target."""
    import oracle
    gkey, opname, F, xdt, gcn = WORKLOADS[workload]
    N, src, dst = graph_of(W, gkey)
    X = W.normal_bf16((N, F), seed=13) if xdt == "bf16" else W.normal_f32((N, F), seed=13)
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, (oracle.SELF_LOOPS | oracle.NORM_SYM) if gcn else 0, want_w=gcn,
                                    threads=threads)
    rop = {"sum": oracle.SUM, "wsum": oracle.WSUM, "mean": oracle.MEAN, "max": oracle.MAX}[opname]
    res = []
    for fc in widths:
        t0 = time.time()
        oracle.aggregate(rop, rp, ci, w, X, f_chunk=fc, form=1, threads=threads)
        dt = time.time() - t0
        res.append({"f_chunk": fc, "seconds": dt, "edge_features_per_s": float(len(ci)) * F / dt, "threads": threads})
        log("checker, chunk-outer, f_chunk=%d: %.2f s" % (fc, dt))
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4-gcn", choices=sorted(WORKLOADS) + ["copy"],
                    help="'copy' runs only the library's plain copy kernel on 1 GiB (profiler calibration)")
    ap.add_argument("--f-chunk", type=int, default=-1,
                    help="chunk width; -1 = let the library pick (GNNAGG_F_CHUNK_AUTO, the default), 0 = one chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--also", default="c4-mean,c5-sum,c5-max,c5-sum-f32,c5-sum-f16,c2-mean,c3-gat,c1-gcn",
                    help="comma list of further workloads measured after the main one and reported under 'also'")
    ap.add_argument("--contiguous", action="store_true",
                    help="keep X and out at a row pitch of exactly F elements instead of line-aligned rows")
    ap.add_argument("--cpu-chunk-sweep", default="",
                    help="comma list of chunk widths: also time the CPU checker in Algorithm 1's chunk-outer order "
                         "on the whole graph of the workload at each width (0 = one chunk); minutes of CPU time")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    import paper_2104_03058_amd as g
    import workloads as W
    g.load_library()

    # plain streaming copy of 1 GiB: the measured HBM copy rate of this device, reported beside the roofline
    probe_bytes = 1 << 30
    p_src = torch.empty(probe_bytes, dtype=torch.uint8, device="cuda").fill_(1)
    p_dst = torch.empty_like(p_src)
    g.gnnagg_copy_probe(p_dst, p_src)
    torch.cuda.synchronize()
    n_probe = max(args.steps, 3) if args.workload == "copy" else 5
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n_probe):
        g.gnnagg_copy_probe(p_dst, p_src)
    e1.record()
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1) / n_probe
    copy_gbs = 2.0 * probe_bytes / (copy_ms * 1e-3) / 1e9
    log("copy probe: 1 GiB in %.3f ms -> %.0f GB/s read+write" % (copy_ms, copy_gbs))
    del p_src, p_dst
    if args.workload == "copy":
        print(json.dumps({"metric": "hbm copy rate", "value": copy_gbs, "unit": "GB/s", "n_gpus": 1,
                          "steps": n_probe, "ms_per_step": copy_ms, "bytes_read": probe_bytes,
                          "bytes_written": probe_bytes, "config": {"workload": "copy"}}), flush=True)
        return

    rec = measure(g, W, torch, args.workload, args.f_chunk, args.steps, args.warmup, not args.no_cpu_baseline,
                  args.cpu_seconds, copy_gbs, not args.contiguous)
    also = []
    for wl in [w for w in args.also.split(",") if w and w != args.workload]:
        r = measure(g, W, torch, wl, args.f_chunk, args.steps, args.warmup, False, 0.0, copy_gbs, not args.contiguous)
        entry = {k: r[k] for k in ("value", "unit", "ms_per_step", "config", "roofline", "setup",
                                   "graph_replay_ms_per_step")}
        med = r["roofline"].get("kernel_ms_median")
        if med:  # the median step is robust against a single stalled step on the microsecond-sized workloads
            entry["ms_median"] = med
            entry["value_median"] = r["value"] * r["ms_per_step"] / med
        also.append(entry)
    rec["also"] = also
    if args.cpu_chunk_sweep:
        rec["cpu_chunk_sweep"] = cpu_chunk_sweep(W, args.workload, [int(v) for v in args.cpu_chunk_sweep.split(",")])
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
