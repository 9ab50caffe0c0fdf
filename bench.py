#!/usr/bin/env python3
"""Benchmark of the fused star-join + prediction hot path on one MI355X.

One "step" = one pass of the method over the workload, inputs resident in HBM:
pre-fusion (lq_project_dims) followed by the join-computation stage
(lq_fused_join_predict).  The headline workload is the 2-layer-MLP star schema
(10M fact rows, dimensions of 1e3/1e4/1e5 rows, MLP 100 -> 64 -> 1, fp32).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      - the dominant kernel (the fused gather kernel) against the HBM roof,
                  from algorithmic bytes / its own event-timed duration
  cpu_baseline  - the fp64 CPU oracle timed on a bounded prefix of the same workload
  stages, materialized, groupby_c3, fused_c4, stream_copy - the other numbers the
                  method is judged by (each timed with events on the launch stream).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def time_call(fn, iters, warmup):
    """Average milliseconds of fn() over `iters` runs, event-timed on the current stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    a, b = _events(iters), _events(iters)
    for i in range(iters):
        a[i].record()
        fn()
        b[i].record()
    torch.cuda.synchronize()
    ts = sorted(x.elapsed_time(y) for x, y in zip(a, b))
    return sum(ts) / len(ts), ts[0], ts[len(ts) // 2]


def graph_time(fn, reps=16, iters=10, warmup=2):
    """Milliseconds per fn() when `reps` calls are recorded into one HIP graph and the graph is replayed:
    the pace of the GPU, for calls so short that the Python caller would otherwise set the pace."""
    import torch
    gs = torch.cuda.Stream()
    with torch.cuda.stream(gs):
        fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=gs):
        for _ in range(reps):
            fn()
    ms, _, _ = time_call(graph.replay, iters, warmup)
    del graph
    return ms / reps


def measured_traffic(key):
    """HBM bytes per launch measured with rocprofv3 counters (committed summary), or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(key)
    except Exception:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--rows", type=int, default=10_000_000, help="fact rows of the headline workload")
    ap.add_argument("--no-extras", action="store_true", help="skip materialised / group-by / skewed legs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only", default="", help="run a single leg for profiling: fused|c1|linear|groupby|groupby16|c4|c5|deep|tree|treesweep|keymap|agg|domain|sweep|sfsweep|materialized|copy")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (no collectives, no sharding); "
                 "run with --gpus 1")

    import torch
    import paper_2306_08367_amd as lq
    from workloads import star as WL

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    out = {}

    # ---------------------------------------------------------------- headline: fused MLP
    n = args.rows
    w = WL.c2_mlp(device=dev, n=n)
    P = [torch.empty((d.shape[0], 64), dtype=torch.float32, device=dev) for d in w.dims]
    Y = torch.empty((n, 1), dtype=torch.float32, device=dev)

    def project():
        lq.lq_project_dims(w.dims, w.weights[0], w.c_f, P=P)

    def fused():
        lq.lq_fused_join_predict(w.X, w.fks, P, w.weights, w.biases, Y=Y)

    def step():
        project()
        fused()

    if args.only in ("", "fused"):
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ea, eb = _events(args.steps), _events(args.steps)
        t0 = time.perf_counter()
        for i in range(args.steps):
            project()
            ea[i].record()
            fused()
            eb[i].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_step = wall * 1e3 / args.steps
        fused_ms = sum(a.elapsed_time(b) for a, b in zip(ea, eb)) / args.steps
        proj_ms, _, _ = time_call(project, 10, 2)
        alg_bytes = 32.0 * n                      # 16 B fact columns + 12 B keys + 4 B output per row
        gather_bytes = 768.0 * n                  # 3 rows of 64 fp32 from the projected tables
        achieved = alg_bytes / (fused_ms * 1e-3) / 1e9
        out.update({
            "metric": "fact rows/s, fused join+predict",
            "value": n * args.steps / wall,
            "unit": "rows/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": "c2_mlp: fused join + 2-layer MLP, fact 10M x 4 fp32, dims "
                                   "1e3/1e4/1e5 x 32 fp32, uniform int32 keys, MLP 100->64 ReLU ->1",
                       "fact_rows": n, "step": "lq_project_dims + lq_fused_join_predict"},
            "roofline": {"bound": "hbm", "kernel": "fused_join_predict (gather + MLP epilogue)",
                         "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBPS,
                         "traffic": measured_traffic("fused_c2"),
                         "algorithmic_bytes_per_row": 32,
                         "note": "768 B/row are gathered from L2/Infinity-Cache-resident projected "
                                 "tables; that gather, not HBM, is the binding roof of this workload",
                         "gather_GBps": gather_bytes / (fused_ms * 1e-3) / 1e9,
                         # counter-measured L2-miss bytes per launch over this run's launch time: what the
                         # fabric (Infinity Cache + HBM) delivered; about 7.4 TB/s is what it sustains here
                         "fabric_GBps": (measured_traffic("fused_c2") or 0.0) / (fused_ms * 1e-3) / 1e9,
                         # reads out of L2 plus fills into it: with every table L2-resident the same kernel
                         # reads 21.9 TB/s out of L2 (768 B/row in 0.35 ms), the rate this sum also comes to
                         "l2_reads_plus_fills_GBps": (gather_bytes + (measured_traffic("fused_c2") or 0.0))
                                                     / (fused_ms * 1e-3) / 1e9},
            "stages": {"project_dims_ms": proj_ms, "fused_join_predict_ms": fused_ms,
                       "fused_rows_per_s": n / (fused_ms * 1e-3)},
        })

    # ---------------------------------------------------------------- CPU oracle baseline
    if args.only == "" and not args.no_cpu:
        from oracle import lq_oracle as O
        sample = min(n, 1 << 23)
        Xs = w.X[:sample].cpu()
        fs = [f[:sample].cpu() for f in w.fks]
        ds = [d.cpu() for d in w.dims]
        Ws = [x.cpu() for x in w.weights]
        threads = min(O.max_threads(), 16, os.cpu_count() or 1)
        t0 = time.perf_counter()
        O.join_predict(Xs, ds, fs, Ws, None, nthreads=threads)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample / dt, "unit": "rows/s", "cores": threads, "kind": "oracle",
                               "sample": f"first {sample} fact rows of the same workload (fp64, "
                                         "tuple materialised then MLP), includes the exact fp32->fp64 "
                                         "widening of the inputs; cost is linear in rows"}

    # ---------------------------------------------------------------- stream-copy yardstick
    if args.only in ("", "copy"):
        nb = 2 << 30
        src = torch.empty(nb, dtype=torch.uint8, device=dev)
        dst = torch.empty(nb, dtype=torch.uint8, device=dev)
        src.zero_()
        ms, _, _ = time_call(lambda: lq.lq_stream_copy(dst, src), 10, 2)
        out["stream_copy"] = {"GBps_read_plus_write": 2 * nb / (ms * 1e-3) / 1e9, "bytes_copied": nb}
        del src, dst

    # ---------------------------------------------------------------- non-fused pipeline
    if (args.only == "" and not args.no_extras) or args.only == "materialized":
        chunk = 1 << 22
        ws_bytes = lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, w.k, w.weights, chunk)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        Ym = torch.empty_like(Y)
        ms, _, _ = time_call(lambda: lq.lq_materialized_join_predict(
            w.X, w.dims, w.fks, w.weights, w.biases, Y=Ym, ws=ws), 3, 1)
        out["materialized"] = {"rows_per_s": n / (ms * 1e-3), "ms": ms, "chunk_rows": chunk}
        if "stages" in out:
            out["materialized"]["fused_speedup"] = ms / (out["stages"]["fused_join_predict_ms"]
                                                        + out["stages"]["project_dims_ms"])
        del ws, Ym
    del w, P, Y
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- tiny linear regression (launch-latency sized)
    if (args.only == "" and not args.no_extras) or args.only == "c1":
        w1 = WL.c1_tiny_linear(device=dev)
        P1 = [torch.empty((d.shape[0], 1), dtype=torch.float32, device=dev) for d in w1.dims]
        Y1 = torch.empty((w1.n, 1), dtype=torch.float32, device=dev)
        ws1 = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, w1.k, w1.weights, 16_384),
                          dtype=torch.uint8, device=dev)
        pus, _, _ = time_call(lambda: lq.lq_project_dims(w1.dims, w1.weights[0], w1.c_f, P=P1), 50, 5)
        fus, _, _ = time_call(lambda: lq.lq_fused_join_predict(w1.X, w1.fks, P1, w1.weights, None, Y=Y1), 50, 5)
        mus, _, _ = time_call(lambda: lq.lq_materialized_join_predict(w1.X, w1.dims, w1.fks, w1.weights, None,
                                                                      Y=Y1, ws=ws1), 50, 5)
        # the same call recorded 32 times into a HIP graph: the pace of the GPU rather than of the Python caller
        gs = torch.cuda.Stream()
        with torch.cuda.stream(gs):
            lq.lq_fused_join_predict(w1.X, w1.fks, P1, w1.weights, None, Y=Y1)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs):
            for _ in range(32):
                lq.lq_fused_join_predict(w1.X, w1.fks, P1, w1.weights, None, Y=Y1)
        gus, _, _ = time_call(graph.replay, 20, 3)
        out["fused_c1"] = {"fact_rows": w1.n, "fused_us": fus * 1e3, "fused_us_in_a_graph": gus * 1e3 / 32,
                           "project_dims_us": pus * 1e3,
                           "materialized_us": mus * 1e3, "rows_per_s": w1.n / (fus * 1e-3),
                           "note": "280 KB of traffic: bound by launch latency; fused_us is paced by the Python caller, "
                                   "fused_us_in_a_graph by the GPU (32 calls per graph)"}

    # ---------------------------------------------------------------- linear regression at scale (the model of Section 3.2)
    if (args.only == "" and not args.no_extras) or args.only == "linear":
        nl = 10_000_000
        cells = {}
        for name, rows, cols in (("c2_star", (1_000, 10_000, 100_000), (32, 32, 32)),
                                 ("dimension_tables_all_in_lds", (1_000, 10_000, 20_000), (32, 32, 32)),
                                 ("four_tables_ssb_sf1_sizes", (2_556, 30_000, 2_000, 200_000), (8, 8, 8, 8))):
            wl = WL.make_predict("linear_" + name, nl, 4, rows, cols, (1,), seed=WL.SEED0 + 800, device=dev, bias=True)
            Pl = lq.lq_project_dims(wl.dims, wl.weights[0], wl.c_f)
            Yl = torch.empty((nl, 1), dtype=torch.float32, device=dev)
            pms, _, _ = time_call(lambda: lq.lq_project_dims(wl.dims, wl.weights[0], wl.c_f, P=Pl), 10, 2)
            fms = graph_time(lambda: lq.lq_fused_join_predict(wl.X, wl.fks, Pl, wl.weights, wl.biases, Y=Yl))
            chunk = 1 << 21
            wsl = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, wl.k, wl.weights, chunk),
                              dtype=torch.uint8, device=dev)
            mms, _, _ = time_call(lambda: lq.lq_materialized_join_predict(wl.X, wl.dims, wl.fks, wl.weights, wl.biases,
                                                                          Y=Yl, ws=wsl), 3, 1)
            bpr = 4 * (4 + len(rows) + 1)
            gbps = bpr * nl / (fms * 1e-3) / 1e9
            cells[name] = {"dim_rows": list(rows), "joined_cols": wl.k, "fused_ms_in_a_graph": fms, "project_dims_ms": pms,
                           "rows_per_s": nl / (fms * 1e-3), "materialized_ms": mms, "fused_speedup": mms / (fms + pms),
                           "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                        "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_row": bpr}}
            del wl, Pl, Yl, wsl
        out["linear_regression"] = {"fact_rows": nl, "fact_cols": 4, "outputs": 1, "cells": cells}
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- LA group-by (SSB-sf1 shape)
    if (args.only == "" and not args.no_extras) or args.only == "groupby":
        g = WL.c3_groupby(device=dev)
        # rotate over several copies of the fact columns so that repeats are not served from cache
        copies = 6
        cols = [([f.clone() for f in g.fks], [m.clone() for m in g.measures]) for _ in range(copies)]
        ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device=dev)
        sums = torch.empty((1, g.G), dtype=torch.int64, device=dev)
        counts = torch.empty((g.G,), dtype=torch.int64, device=dev)
        it = [0]

        def gb():
            fk, me = cols[it[0] % copies]
            it[0] += 1
            lq.lq_masked_groupby_sum(fk, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None, me,
                                     sums=sums, counts=counts, ws=ws)
        ms, mn, med = time_call(gb, 30, 6)

        def gb_reuse():                                  # dimension side already encoded in ws
            fk, me = cols[it[0] % copies]
            it[0] += 1
            lq.lq_masked_groupby_sum(fk, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None, me,
                                     sums=sums, counts=counts, ws=ws, flags=lq.LQ_REUSE_SIDE_TABLES)
        rms, _, _ = time_call(gb_reuse, 30, 6)
        gbps = 20.0 * g.n / (ms * 1e-3) / 1e9
        out["groupby_c3"] = {"rows_per_s": g.n / (ms * 1e-3), "ms": ms, "ms_min": mn, "fact_rows": g.n,
                             "ms_reuse_side_tables": rms,
                             "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                                          "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                                          "algorithmic_bytes_per_row": 20,
                                          "traffic": measured_traffic("groupby_c3")}}
        del g, cols
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- skewed linear model (HBM-bound)
    if (args.only == "" and not args.no_extras) or args.only == "c4":
        n4 = 100_000_000
        w4 = WL.c4_skewed(device=dev, n=n4)
        P4 = [torch.empty((d.shape[0], 4), dtype=torch.float32, device=dev) for d in w4.dims]
        Y4 = torch.empty((n4, 4), dtype=torch.float32, device=dev)
        pms, _, _ = time_call(lambda: lq.lq_project_dims(w4.dims, w4.weights[0], w4.c_f, P=P4), 5, 1)
        ms, mn, _ = time_call(lambda: lq.lq_fused_join_predict(w4.X, w4.fks, P4, w4.weights, None, Y=Y4), 10, 2)
        gbps = 56.0 * n4 / (ms * 1e-3) / 1e9
        m4 = 1 << 23                                  # non-fused pipeline on a slice: T of all rows is 106 GB
        ws4 = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, w4.k, w4.weights, 1 << 21),
                          dtype=torch.uint8, device=dev)
        Ym4 = torch.empty((m4, 4), dtype=torch.float32, device=dev)
        mms4, _, _ = time_call(lambda: lq.lq_materialized_join_predict(w4.X[:m4], w4.dims, [f[:m4] for f in w4.fks],
                                                                       w4.weights, None, Y=Ym4, ws=ws4), 2, 1)
        out["fused_c4"] = {"rows_per_s": n4 / (ms * 1e-3), "ms": ms, "project_dims_ms": pms, "fact_rows": n4,
                           "materialized_rows_per_s": m4 / (mms4 * 1e-3),
                           "fused_speedup": (mms4 / m4) / ((ms + pms) / n4),
                           "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                                        "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                                        "algorithmic_bytes_per_row": 56,
                                        "traffic": measured_traffic("fused_c4")},
                           "project_dims_GBps": 2 * 1_000_000 * 128 * 4 / (pms * 1e-3) / 1e9}
        del w4, P4, Y4, ws4, Ym4
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- wide bf16 MLP (cache-gather bound)
    if (args.only == "" and not args.no_extras) or args.only == "c5":
        n5 = 50_000_000
        w5 = WL.c5_wide_bf16(device=dev, n=n5)
        P5 = [torch.empty((d.shape[0], 256), dtype=torch.bfloat16, device=dev) for d in w5.dims]
        Y5 = torch.empty((n5, 16), dtype=torch.bfloat16, device=dev)
        pms, _, _ = time_call(lambda: lq.lq_project_dims(w5.dims, w5.weights[0], 0, P=P5), 5, 1)
        ms, mn, _ = time_call(lambda: lq.lq_fused_join_predict(None, w5.fks, P5, w5.weights, None, Y=Y5), 5, 1)
        m5 = 1 << 22                                  # non-fused pipeline on a slice: T of all rows is 102 GB
        ws5 = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, w5.k, w5.weights, 1 << 20),
                          dtype=torch.uint8, device=dev)
        fk5 = [f[:m5] for f in w5.fks]
        Ym5 = torch.empty((m5, 16), dtype=torch.bfloat16, device=dev)
        mms, _, _ = time_call(lambda: lq.lq_materialized_join_predict(None, w5.dims, fk5, w5.weights, None,
                                                                      Y=Ym5, ws=ws5), 2, 1)
        out["fused_c5"] = {"rows_per_s": n5 / (ms * 1e-3), "ms": ms, "project_dims_ms": pms, "fact_rows": n5,
                           "dtype": "bf16", "gather_GBps": 2048.0 * n5 / (ms * 1e-3) / 1e9,
                           "hbm_GBps_algorithmic": 48.0 * n5 / (ms * 1e-3) / 1e9,
                           "materialized_rows_per_s": m5 / (mms * 1e-3),
                           "fused_speedup": (mms / m5) / ((ms + pms) / n5)}
        del w5, P5, Y5, ws5, Ym5
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- deeper models (later layers on the matrix cores)
    if (args.only == "" and not args.no_extras) or args.only == "deep":
        nd = 4_000_000
        cells = {}
        for name, dt, rows, cols, c_f, layers, sig in (
                ("f32_c2star_64_64_1", torch.float32, (1_000, 10_000, 100_000), (32, 32, 32), 4, (64, 64, 1), 0.1),
                ("f32_c2star_128_64_1", torch.float32, (1_000, 10_000, 100_000), (32, 32, 32), 4, (128, 64, 1), 0.1),
                ("f32_c2star_64_16", torch.float32, (1_000, 10_000, 100_000), (32, 32, 32), 4, (64, 16), 0.1),
                ("bf16_c5star_256_64_16", torch.bfloat16, (10_000,) * 4, (64,) * 4, 0, (256, 64, 16), 0.06)):
            wd = WL.make_predict(name, nd, c_f, rows, cols, layers, seed=WL.SEED0 + 950, dtype=dt, device=dev,
                                 w_sigma=[sig] * len(layers))
            Pd = lq.lq_project_dims(wd.dims, wd.weights[0], c_f, p_dtype=dt)
            Yd = torch.empty((nd, layers[-1]), dtype=dt, device=dev)
            ms, _, _ = time_call(lambda: lq.lq_fused_join_predict(wd.X, wd.fks, Pd, wd.weights, None, Y=Yd), 10, 2)
            wsd = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, wd.k, wd.weights, 1 << 20),
                              dtype=torch.uint8, device=dev)
            mms, _, _ = time_call(lambda: lq.lq_materialized_join_predict(wd.X, wd.dims, wd.fks, wd.weights, None,
                                                                          Y=Yd, ws=wsd), 2, 1)
            later_flop = 2.0 * sum(a * b for a, b in zip(layers[:-1], layers[1:])) * nd
            cells[name] = {"fused_ms": round(ms, 4), "rows_per_s": nd / (ms * 1e-3),
                           "later_layers_TFLOPs": later_flop / (ms * 1e-3) / 1e12,
                           "gather_GBps": len(rows) * layers[0] * wd.dims[0].element_size() * nd / (ms * 1e-3) / 1e9,
                           "materialized_ms": round(mms, 3), "fused_speedup": mms / ms}
            del wd, Pd, Yd, wsd
        torch.cuda.empty_cache()
        out["deeper_models"] = {"fact_rows": nd, "cells": cells}

    # ---------------------------------------------------------------- group-by at 16x the fact rows
    if (args.only == "" and not args.no_extras) or args.only == "groupby16":
        g = WL.c3_groupby(device=dev, n=96_000_000, dim_rows=(2_556, 480_000, 32_000, 1_000_000))
        ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device=dev)
        sums = torch.empty((1, g.G), dtype=torch.int64, device=dev)
        counts = torch.empty((g.G,), dtype=torch.int64, device=dev)
        ms, mn, _ = time_call(lambda: lq.lq_masked_groupby_sum(g.fks, g.dim_rows, g.dim_mask, g.dim_code,
                                                               g.group_card, None, g.measures, sums=sums,
                                                               counts=counts, ws=ws), 10, 2)
        gbps = 20.0 * g.n / (ms * 1e-3) / 1e9
        out["groupby_sf16_shape"] = {"rows_per_s": g.n / (ms * 1e-3), "ms": ms, "fact_rows": g.n,
                                     "dim_rows": list(g.dim_rows),
                                     "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                                                  "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                                                  "algorithmic_bytes_per_row": 20}}
        del g

    # ---------------------------------------------------------------- decision tree (setting 1, sf 8)
    if (args.only == "" and not args.no_extras) or args.only == "tree":
        nt = 4_800_000
        wt = WL.make_predict("tree_s1_sf8", nt, 0, (80_000, 16_000, 2_555), (43, 43, 42), (1,),
                             seed=WL.SEED0 + 700, device=dev)
        tree = WL.make_tree(128, 64, WL.SEED0 + 701)
        tf, tt, tH = tree.feature.to(dev), tree.threshold.to(dev), tree.H.to(dev)
        tables, target = lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH)
        pms, _, _ = time_call(lambda: lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH), 5, 1)
        ms, mn, _ = time_call(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH), 20, 3)
        mms, _, _ = time_call(lambda: lq.lq_materialized_join_tree(None, wt.dims, wt.fks, tf, tt, tH,
                                                                   chunk_rows=1 << 20), 2, 1)
        gbps = 16.0 * nt / (ms * 1e-3) / 1e9
        # leaf masks: the same tables compressed to one bit per leaf, AND instead of sum-and-compare
        masks = lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH)
        cms, _, _ = time_call(lambda: lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH), 5, 1)
        kms, _, _ = time_call(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH), 20, 3)
        gms = graph_time(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH))
        kgms = graph_time(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH))
        kgbps = 16.0 * nt / (kgms * 1e-3) / 1e9
        out["fused_tree"] = {"rows_per_s": nt / (ms * 1e-3), "ms": ms, "project_ms": pms, "fact_rows": nt,
                             "leaves": 64, "nodes": 63, "joined_cols": 128,
                             "materialized_rows_per_s": nt / (mms * 1e-3),
                             "fused_speedup": mms / (ms + pms),
                             "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                          "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_row": 16,
                                          "gather_GBps": 192.0 * nt / (ms * 1e-3) / 1e9},
                             "ms_in_a_graph": gms,
                             "leaf_masks": {"rows_per_s": nt / (kgms * 1e-3), "ms": kms, "ms_in_a_graph": kgms,
                                            "compress_ms": cms,
                                            "fused_speedup": mms / (kms + pms + cms),
                                            "roofline": {"bound": "hbm", "achieved": kgbps, "peak": HBM_PEAK_GBPS,
                                                         "unit": "GB/s", "frac": kgbps / HBM_PEAK_GBPS,
                                                         "algorithmic_bytes_per_row": 16}}}
        del wt, tables, masks
        # the same tree size with 8 of the 128 joined columns in the fact table itself: their nodes are
        # evaluated per fact row in the join stage
        wf = WL.make_predict("tree_s1_sf8_fact", nt, 8, (80_000, 16_000, 2_555), (40, 40, 40), (1,),
                             seed=WL.SEED0 + 702, device=dev)
        tables, target = lq.lq_tree_project_dims(wf.dims, 8, tf, tt, tH)
        masks = lq.lq_tree_compress_tables(wf.dims, tables, tf, tt, tH, c_f=8)
        fmask = lq.lq_tree_fact_masks(8, tf, tt, tH)
        fcnt = int(fmask[:4].view(torch.int32).item())
        fms, _, _ = time_call(lambda: lq.lq_fused_join_tree(wf.X, wf.fks, tables, target, tf, tt, tH), 5, 1)
        fkms = graph_time(lambda: lq.lq_fused_join_tree_masks(wf.fks, masks, tf, tt, tH, X=wf.X, fact_masks=fmask))
        fmms, _, _ = time_call(lambda: lq.lq_materialized_join_tree(wf.X, wf.dims, wf.fks, tf, tt, tH,
                                                                    chunk_rows=1 << 20), 2, 1)
        fgbps = 48.0 * nt / (fkms * 1e-3) / 1e9
        out["fused_tree"]["with_fact_columns"] = {
            "fact_cols": 8, "nodes_on_fact_cols": fcnt, "byte_tables_ms": fms, "leaf_masks_ms_in_a_graph": fkms,
            "materialized_ms": fmms, "fused_speedup_join_stage": fmms / fkms,
            "roofline": {"bound": "hbm", "achieved": fgbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": fgbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_row": 48}}
        del wf, tables, masks, fmask

    # ---------------------------------------------------------------- trees of growing size (only on request)
    # cardinality settings 1 (large dimension tables, sf 4) and 2 (small ones), leaves 8 .. 2,048:
    # where the pre-fusion stage starts to dominate (Section 4.4, the tree experiments)
    if args.only == "treesweep":
        cells = {}
        for setting, nt, rows in (("setting1_sf4", 2_400_000, (40_000, 8_000, 2_555)),
                                  ("setting2", 2_400_000, (1_000, 500, 2_555))):
            wt = WL.make_predict("tree_sweep", nt, 0, rows, (43, 43, 42), (1,), seed=WL.SEED0 + 720, device=dev)
            for leaves in (8, 64, 256, 1024, 2048):
                tree = WL.make_tree(128, leaves, WL.SEED0 + 721 + leaves)
                tf, tt, tH = tree.feature.to(dev), tree.threshold.to(dev), tree.H.to(dev)
                tables, target = lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH)
                pms, _, _ = time_call(lambda: lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH), 3, 1)
                ms, _, _ = time_call(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH), 5, 1)
                mms, _, _ = time_call(lambda: lq.lq_materialized_join_tree(None, wt.dims, wt.fks, tf, tt, tH,
                                                                           chunk_rows=1 << 19), 1, 1)
                masks = lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH)
                cms, _, _ = time_call(lambda: lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH), 3, 1)
                kms, _, _ = time_call(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH), 5, 1)
                gms = graph_time(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH), 8, 5, 1)
                kgms = graph_time(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH), 8, 5, 1)
                cells[f"{setting}_l{leaves}"] = {"fused_ms": round(ms, 4), "prefusion_ms": round(pms, 4),
                                                 "materialized_ms": round(mms, 3),
                                                 "speedup_join_stage": round(mms / ms, 1),
                                                 "speedup_with_prefusion": round(mms / (ms + pms), 1),
                                                 "fused_ms_in_a_graph": round(gms, 4),
                                                 "masks_fused_ms": round(kms, 4), "masks_fused_ms_in_a_graph": round(kgms, 4),
                                                 "masks_compress_ms": round(cms, 4),
                                                 "masks_speedup_join_stage": round(mms / kms, 1),
                                                 "masks_speedup_with_prefusion": round(mms / (kms + pms + cms), 1)}
                del tables, masks
            del wt
            torch.cuda.empty_cache()
        out["tree_sweep"] = {"fact_rows": 2_400_000, "joined_cols": 128, "cells": cells}

    # ---------------------------------------------------------------- key -> row mapping (SSB sf1 shape)
    if (args.only == "" and not args.no_extras) or args.only == "keymap":
        nk = 6_000_000
        gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 900)
        res = {}
        tot_ms = 0.0
        tot_dense = 0.0
        for r in (2_556, 30_000, 2_000, 200_000):
            # sparse unique keys: a random subset of 0 .. 8r, shuffled
            keys_S = torch.randperm(8 * r, generator=gen, device=dev)[:r].to(torch.int32)
            fact = keys_S[torch.randint(0, r, (nk,), generator=gen, device=dev)]
            table = lq.lq_keymap_build(keys_S)
            fk = torch.empty(nk, dtype=torch.int32, device=dev)
            bms, _, _ = time_call(lambda: lq.lq_keymap_build(keys_S), 5, 1)
            lms, _, _ = time_call(lambda: lq.lq_keymap_lookup(table, fact, fk=fk), 20, 3)
            res[str(r)] = {"build_ms": bms, "lookup_ms": lms, "lookup_GBps": 8.0 * nk / (lms * 1e-3) / 1e9}
            tot_ms += lms
            # surrogate keys 1..r in shuffled row order: the dense range makes the map a direct array
            keys_D = (torch.randperm(r, generator=gen, device=dev) + 1).to(torch.int32)
            fact_D = keys_D[torch.randint(0, r, (nk,), generator=gen, device=dev)]
            table_D = lq.lq_keymap_build(keys_D)
            dbms, _, _ = time_call(lambda: lq.lq_keymap_build(keys_D), 5, 1)
            dlms, _, _ = time_call(lambda: lq.lq_keymap_lookup(table_D, fact_D, fk=fk), 20, 3)
            res[str(r)].update({"dense_build_ms": dbms, "dense_lookup_ms": dlms,
                                "dense_lookup_GBps": 8.0 * nk / (dlms * 1e-3) / 1e9})
            tot_dense += dlms
        gbps = 4 * 8.0 * nk / (tot_ms * 1e-3) / 1e9
        out["keymap_ssb_sf1"] = {"fact_rows": nk, "rows_per_s_all_4_columns": nk / (tot_ms * 1e-3),
                                 "dense_keys_rows_per_s_all_4_columns": nk / (tot_dense * 1e-3), "per_dimension": res,
                                 "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                              "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_row": 8}}

    # ---------------------------------------------------------------- wider aggregate (1 join, fact predicates, SUM(a*b))
    if (args.only == "" and not args.no_extras) or args.only == "agg":
        na = 6_000_000
        gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 950)
        ri = lambda lo, hi: torch.randint(lo, hi, (na,), generator=gen, device=dev, dtype=torch.int32)
        fk = ri(0, 2_556)
        price, disc, qty = ri(1, 100_001), ri(0, 11), ri(1, 51)
        dmask = (torch.arange(2_556, device=dev) % 7 == 3).to(torch.uint8)
        call = lambda: lq.lq_groupby_agg([fk], [2_556], [dmask], [None], [1], [(disc, 1, 3), (qty, 1, 24)],
                                         [("mul", price, disc)], want=("sum", "count"))
        ms, mn, _ = time_call(call, 20, 3)
        gbps = 16.0 * na / (ms * 1e-3) / 1e9
        out["agg_one_join"] = {"rows_per_s": na / (ms * 1e-3), "ms": ms, "fact_rows": na,
                               "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                            "frac": gbps / HBM_PEAK_GBPS, "algorithmic_bytes_per_row": 16}}

    # ---------------------------------------------------------------- group discovery + ORDER BY (query set-up / tail)
    if (args.only == "" and not args.no_extras) or args.only == "domain":
        gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 960)
        rd = 1_400_000                                                       # part dimension at sf 16
        a5 = torch.randint(0, 5, (rd,), generator=gen, device=dev, dtype=torch.int32) * 11 + 3
        b25 = a5 * 5 + torch.randint(0, 5, (rd,), generator=gen, device=dev, dtype=torch.int32)
        dms, _, _ = time_call(lambda: lq.lq_group_domain([a5, b25]), 10, 2)   # includes its one host wait
        Gd = 7 * 25
        cnt = torch.randint(0, 1000, (Gd,), generator=gen, device=dev, dtype=torch.int64)
        sm = torch.randint(0, 1 << 40, (1, Gd), generator=gen, device=dev, dtype=torch.int64)
        o_buf = torch.empty(8192, dtype=torch.int32, device=dev)
        n_buf = torch.empty(1, dtype=torch.int32, device=dev)
        oms, _, _ = time_call(lambda: lq.lq_order_groups([7, 25], sm, cnt, [(0, 0, False), (1, 0, True)],
                                                         order=o_buf, n_out=n_buf), 20, 3)
        cnt8 = torch.randint(0, 3, (8192,), generator=gen, device=dev, dtype=torch.int64)
        sm8 = torch.randint(0, 1 << 40, (1, 8192), generator=gen, device=dev, dtype=torch.int64)
        oms8, _, _ = time_call(lambda: lq.lq_order_groups([64, 128], sm8, cnt8, [(1, 0, True)],
                                                          order=o_buf, n_out=n_buf), 20, 3)
        out["group_domain_and_order"] = {"group_domain_ms": dms, "dim_rows": rd, "columns": 2, "groups": 25,
                                         "order_175_groups_ms": oms, "order_8192_groups_ms": oms8}

    # ---------------------------------------------------------------- k x l sweep (setting 1, sf 4, linear operator)
    if (args.only == "" and not args.no_extras) or args.only == "sweep":
        ns = 2_400_000
        rows_s = (60_000, 8_000, 2_555)
        split = {16: (8, 4, 4), 32: (12, 12, 8), 64: (24, 20, 20), 128: (44, 44, 40)}
        sweep = {}
        ws_s = None
        for k_in, cols in split.items():
            for l_out in (2, 4, 8, 16, 32, 64, 128):
                wk = WL.make_predict("sweep", ns, 0, rows_s, cols, (l_out,), seed=WL.SEED0 + 1000 + k_in, device=dev)
                Pk = lq.lq_project_dims(wk.dims, wk.weights[0], 0)
                Yk = torch.empty((ns, l_out), dtype=torch.float32, device=dev)
                fms, _, _ = time_call(lambda: lq.lq_fused_join_predict(None, wk.fks, Pk, wk.weights, None, Y=Yk), 5, 1)
                pms, _, _ = time_call(lambda: lq.lq_project_dims(wk.dims, wk.weights[0], 0, P=Pk), 3, 1)
                need = lq.lq_workspace_bytes(lq.binding.LQ_CALL_MATERIALIZED, k_in, wk.weights, 1 << 21)
                if ws_s is None or ws_s.numel() < need:
                    ws_s = torch.empty(need, dtype=torch.uint8, device=dev)
                mms, _, _ = time_call(lambda: lq.lq_materialized_join_predict(None, wk.dims, wk.fks, wk.weights, None,
                                                                              Y=Yk, ws=ws_s), 2, 1)
                sweep[f"k{k_in}_l{l_out}"] = {"fused_ms": round(fms, 4), "prefusion_ms": round(pms, 4),
                                              "materialized_ms": round(mms, 4), "speedup": round(mms / fms, 2),
                                              "k_over_l": k_in / l_out}
        out["sweep_setting1_sf4"] = {"fact_rows": ns, "dim_rows": list(rows_s), "cells": sweep}

    # ---------------------------------------------------------------- group-by over scale factors 1..16
    # (only on request: the table cardinalities grow as in Section 4.1; rows/s over sf is the scaling curve)
    if args.only == "sfsweep":
        import math
        cells = {}
        for sf in (1, 2, 4, 8, 16):
            rows_sf = (2_556, 30_000 * sf, 2_000 * sf, int(200_000 * (1 + math.log2(sf))))
            g = WL.c3_groupby(device=dev, n=6_000_000 * sf, dim_rows=rows_sf)
            copies = max(1, 8 // sf)                      # rotate copies while the columns would fit in cache
            cols = [([f.clone() for f in g.fks], [m.clone() for m in g.measures]) for _ in range(copies)]
            ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device=dev)
            sums = torch.empty((1, g.G), dtype=torch.int64, device=dev)
            counts = torch.empty((g.G,), dtype=torch.int64, device=dev)
            it = [0]

            def gb():
                fk, me = cols[it[0] % copies]
                it[0] += 1
                lq.lq_masked_groupby_sum(fk, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None, me,
                                         sums=sums, counts=counts, ws=ws)
            ms, mn, _ = time_call(gb, 20, 4)
            cells[f"sf{sf}"] = {"fact_rows": g.n, "dim_rows": list(rows_sf), "ms": round(ms, 4),
                                "rows_per_s": g.n / (ms * 1e-3), "GBps": 20.0 * g.n / (ms * 1e-3) / 1e9}
            del g, cols, ws
            torch.cuda.empty_cache()
        out["groupby_sf_sweep"] = cells

    print(json.dumps(out))


if __name__ == "__main__":
    main()
