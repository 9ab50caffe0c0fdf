#!/usr/bin/env python3
"""Benchmark of the fused star-join + prediction hot path and the LA group-by on one MI355X.

One "step" = one pass of the method over the workload, inputs resident in HBM:
pre-fusion (lq_project_dims) followed by the join-computation stage
(lq_fused_join_predict).  The headline workload is the 2-layer-MLP star schema
(10M fact rows, dimensions of 1e3/1e4/1e5 rows, MLP 100 -> 64 -> 1, fp32).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      - the dominant kernel (the fused gather kernel) against the HBM roof, from algorithmic
                  bytes / its own event-timed duration, next to the cache-gather yardstick that binds it
  cpu_baseline  - the fp64 CPU oracle timed on a bounded prefix of the same workload (all host threads)
  yardsticks    - what this GPU delivers for a plain copy, a read sweep (HBM / Infinity Cache) and random row
                  gathers: the measured roofs the per-configuration cells are quoted against
  one cell per configuration / leg (each event-timed on the launch stream: mean, median and min; the
  non-fused pipeline beside the fused one; the CPU oracle at 1 thread and at all threads under "cpu")
  summary       - right after the contract's keys: the five named configurations in a few numbers each
"""
from __future__ import annotations

import argparse
import json
import math
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
    """(mean, min, median) milliseconds of fn() over `iters` runs, event-timed on the current stream."""
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


def tstats(t, prefix=""):
    """The three figures of time_call as a dict."""
    mean, mn, med = t
    return {prefix + "ms": mean, prefix + "ms_median": med, prefix + "ms_min": mn}


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
    _, _, med = time_call(graph.replay, iters, warmup)
    del graph
    return med / reps


def measured_traffic(key):
    """HBM bytes per launch measured with rocprofv3 counters (committed summary), or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(key)
    except Exception:
        return None


def hbm_roofline(bytes_per_row, rows, ms, **extra):
    gbps = bytes_per_row * rows / (ms * 1e-3) / 1e9
    d = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
         "algorithmic_bytes_per_row": bytes_per_row}
    d.update(extra)
    return d


def cpu_threads():
    from oracle import lq_oracle as O
    return max(1, min(O.max_threads(), 16, os.cpu_count() or 1))


def cpu_predict(w, rows_all, rows_one):
    """Oracle rows/s on a prefix of a prediction workload: all host threads, then one thread."""
    from oracle import lq_oracle as O
    nt = cpu_threads()
    out = {"kind": "oracle (fp64, joined tuple materialised row by row, then the layers)", "host_threads_available": os.cpu_count()}
    ds = [d.cpu() for d in w.dims]
    Ws = [x.cpu() for x in w.weights]
    bs = None if w.biases is None else [None if b is None else b.cpu() for b in w.biases]
    for label, threads, rows in (("all_threads", nt, rows_all), ("one_thread", 1, rows_one)):
        rows = min(rows, w.n)
        Xs = None if w.X is None else w.X[:rows].cpu()
        fs = [f[:rows].cpu() for f in w.fks]
        t0 = time.perf_counter()
        O.join_predict(Xs, ds, fs, Ws, bs, nthreads=threads)
        dt = time.perf_counter() - t0
        out[label] = {"rows_per_s": rows / dt, "threads": threads, "sample_rows": rows, "seconds": dt,
                      "extrapolated": rows < w.n}
    return out


def cpu_groupby(g):
    from oracle import lq_oracle as O
    nt = cpu_threads()
    out = {"kind": "oracle (int64, tuple by tuple)", "host_threads_available": os.cpu_count()}
    cpu = lambda ts: [None if t is None else t.cpu() for t in ts]
    fks, masks, codes, meas = cpu(g.fks), cpu(g.dim_mask), cpu(g.dim_code), cpu(g.measures)
    for label, threads in (("all_threads", nt), ("one_thread", 1)):
        t0 = time.perf_counter()
        O.groupby_sum(fks, g.dim_rows, masks, codes, g.group_card, None, meas, nthreads=threads)
        dt = time.perf_counter() - t0
        out[label] = {"rows_per_s": g.n / dt, "threads": threads, "sample_rows": g.n, "seconds": dt, "extrapolated": False}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--rows", type=int, default=10_000_000, help="fact rows of the headline workload")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload and its CPU baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip every CPU oracle baseline")
    ap.add_argument("--only", default="", help="run a single leg for profiling: fused|yardsticks|c1|linear|groupby|groupby_many|"
                    "groupby16|c4|c5|deep|wide_models|tree|treesweep|keymap|agg|domain|sweep|setting2|sfsweep|materialized")
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
    MAT = lq.binding.LQ_CALL_MATERIALIZED
    do_cpu = not args.no_cpu and args.only == ""

    def want(leg):
        return (args.only == "" and not args.no_extras) or args.only == leg

    def guarded(name, fn):
        """Runs one leg; a failure is recorded in its cell and reported on stderr, the other legs still run."""
        try:
            fn()
        except Exception as e:  # noqa: BLE001
            out[name] = {"error": f"{type(e).__name__}: {e}"}
            print(f"bench.py: leg {name} failed: {e}", file=sys.stderr)
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- yardsticks (measured roofs)
    yard = {}

    def leg_yardsticks():
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        nb = 2 << 30
        src = torch.empty(nb, dtype=torch.uint8, device=dev)
        dst = torch.empty(nb, dtype=torch.uint8, device=dev)
        src.zero_()
        t = time_call(lambda: lq.lq_stream_copy(dst, src), 10, 2)
        yard["stream_copy_GBps_read_plus_write"] = 2 * nb / (t[2] * 1e-3) / 1e9
        t = time_call(lambda: lq.lq_yardstick_read(src, 1, sink), 10, 2)
        yard["hbm_read_GBps"] = nb / (t[2] * 1e-3) / 1e9                       # 2 GiB, read once
        small = src[:64 << 20]
        t = time_call(lambda: lq.lq_yardstick_read(small, 32, sink), 10, 2)
        yard["infinity_cache_read_GBps"] = 32 * (64 << 20) / (t[2] * 1e-3) / 1e9   # 64 MiB, read 32 times per launch
        tiny = src[:2 << 20]
        t = time_call(lambda: lq.lq_yardstick_read(tiny, 1024, sink), 10, 2)
        yard["l2_read_GBps"] = 1024 * (2 << 20) / (t[2] * 1e-3) / 1e9              # 2 MiB, read 1,024 times per launch
        del dst
        # random row gathers, row numbers hashed in the kernel (no stream beside them)
        ng = 30_000_000
        for name, table_bytes, row_bytes in (("gather_256B_rows_of_25.6MB", 25_600_000, 256),     # C2's largest projected table
                                             ("gather_256B_rows_of_2.56MB", 2_560_000, 256),      # C2's middle table: fits L2
                                             ("gather_256B_rows_of_0.256MB", 256_000, 256),       # C2's smallest table
                                             ("gather_512B_rows_of_20.5MB", 20_480_000, 512),     # C5's four tables together
                                             ("gather_16B_rows_of_32MB", 32_000_000, 16),         # C4's two tables together
                                             ("gather_16B_rows_of_2MB", 2_000_000, 16)):
            tab = src[:table_bytes]
            t = time_call(lambda: lq.lq_yardstick_gather(tab, row_bytes, ng, sink), 10, 2)
            yard[name + "_GBps"] = ng * row_bytes / (t[2] * 1e-3) / 1e9
            yard[name + "_Grows_per_s"] = ng / (t[2] * 1e-3) / 1e9
        # fp32 matrix instructions alone and with vector instructions between them (three wavefronts per SIMD)
        msink = torch.empty(256 * 8 * 256, dtype=torch.float32, device=dev)
        it_m = 2000
        mflop = 256 * 4 * 3 * it_m * 16 * 2048.0                      # SIMDs x wavefronts x iterations x 16 x (16*16*4*2)
        tm = {nv: time_call(lambda: lq.lq_yardstick_matrix(nv, 3, it_m, msink), 10, 2)[2] for nv in (0, 64, 128)}
        yard["fp32_matrix_TFLOPs"] = mflop / (tm[0] * 1e-3) / 1e12
        yard["fp32_matrix_TFLOPs_with_4_vector_ops_per_matrix_op"] = mflop / (tm[64] * 1e-3) / 1e12
        yard["fp32_matrix_TFLOPs_with_8_vector_ops_per_matrix_op"] = mflop / (tm[128] * 1e-3) / 1e12
        # time the vector instructions add, as a fraction of what they take alone (4 cycles each at 2.4 GHz)
        alone = 3 * it_m * 128 * 4 / 2.4e9 * 1e3
        yard["vector_time_not_hidden_by_matrix_ops_frac"] = (tm[128] - tm[0]) / alone
        del msink
        yard["note"] = ("medians of 10 launches; copy and HBM read over 2 GiB, Infinity Cache read = 64 MiB read 32 times in one "
                        "launch, L2 read = 2 MiB read 1,024 times; gathers: 3e7 uniform random rows per launch, a row fetched by "
                        "adjacent lanes as one run, eight rows in flight per lane, nothing written; fp32 matrix: 16x16x4 "
                        "instructions, three wavefronts per SIMD, 16 per iteration followed by 0 / 64 / 128 independent vector "
                        "multiply-adds")
        out["yardsticks"] = yard
        out["stream_copy"] = {"GBps_read_plus_write": yard["stream_copy_GBps_read_plus_write"], "bytes_copied": nb}

    if args.only in ("", "yardsticks", "fused", "c4", "c5", "deep", "keymap"):
        guarded("yardsticks", leg_yardsticks)

    # ---------------------------------------------------------------- headline: fused MLP (C2)
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
        fts = sorted(a.elapsed_time(b) for a, b in zip(ea, eb))
        fused_ms = sum(fts) / len(fts)
        proj = time_call(project, 10, 2)
        alg_bytes = 32.0 * n                      # 16 B fact columns + 12 B keys + 4 B output per row
        gather_bytes = 768.0 * n                  # 3 rows of 64 fp32 from the projected tables
        achieved = alg_bytes / (fused_ms * 1e-3) / 1e9
        gather_gbps = gather_bytes / (fused_ms * 1e-3) / 1e9
        # the same three gathers with nothing else, one table after the other (uniform random 256-byte rows)
        rates = [yard.get(f"gather_256B_rows_of_{mb}MB_Grows_per_s") for mb in ("25.6", "2.56", "0.256")]
        roof_ms = sum(n / (r * 1e9) * 1e3 for r in rates) if all(rates) else None
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
                       "fact_rows": n, "step": "lq_project_dims + lq_fused_join_predict",
                       "inputs": "320 MB of fact columns, not rotated between steps (above the 256 MB Infinity Cache)"},
            "roofline": {"bound": "hbm", "kernel": "fused_join_predict (gather + MLP epilogue)",
                         "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBPS,
                         "traffic": measured_traffic("fused_c2"),
                         "algorithmic_bytes_per_row": 32,
                         "note": "768 B/row are gathered from L2/Infinity-Cache-resident projected "
                                 "tables; that gather, not HBM, is the binding roof of this workload: "
                                 "gather_frac_of_yardstick = time of the bare gathers (yardstick kernel, one table after "
                                 "the other) / time of this kernel",
                         "gather_GBps": gather_gbps,
                         # the gather yardstick on tables of the three sizes, run one after the other
                         "gather_yardstick_ms": roof_ms,
                         "gather_frac_of_yardstick": (roof_ms / fused_ms) if roof_ms else None,
                         # counter-measured L2-miss bytes per launch over this run's launch time: what the
                         # fabric (Infinity Cache + HBM) delivered
                         "fabric_GBps": (measured_traffic("fused_c2") or 0.0) / (fused_ms * 1e-3) / 1e9,
                         "l2_reads_plus_fills_GBps": (gather_bytes + (measured_traffic("fused_c2") or 0.0))
                                                     / (fused_ms * 1e-3) / 1e9},
            "stages": {"project_dims_ms": proj[0], "project_dims_ms_median": proj[2],
                       "fused_join_predict_ms": fused_ms, "fused_join_predict_ms_median": fts[len(fts) // 2],
                       "fused_join_predict_ms_min": fts[0], "fused_rows_per_s": n / (fused_ms * 1e-3)},
        })

    # ---------------------------------------------------------------- CPU oracle baseline (C2)
    if do_cpu:
        c2cpu = cpu_predict(w, 1 << 23, 1 << 20)
        a = c2cpu["all_threads"]
        out["cpu_baseline"] = {"value": a["rows_per_s"], "unit": "rows/s", "cores": a["threads"], "kind": "oracle",
                               "sample": f"first {a['sample_rows']} fact rows of the same workload (fp64, tuple materialised "
                                         "then MLP), includes the exact fp32->fp64 widening of the inputs; cost is linear in "
                                         "rows; one thread: see cpu_c2",
                               "host_threads_available": os.cpu_count()}
        out["cpu_c2"] = c2cpu

    # ---------------------------------------------------------------- non-fused pipeline (C2)
    def leg_materialized():
        chunk = 1 << 22
        ws = torch.empty(lq.lq_workspace_bytes(MAT, w.k, w.weights, chunk), dtype=torch.uint8, device=dev)
        Ym = torch.empty_like(Y)
        t = time_call(lambda: lq.lq_materialized_join_predict(w.X, w.dims, w.fks, w.weights, w.biases, Y=Ym, ws=ws), 5, 1)
        # per row: X and keys in, the joined tuple T written and read back, the hidden layer written and read back, Y out
        l1m = int(w.weights[0].shape[1])
        bpr = 4 * (w.c_f + len(w.fks)) + 2 * 4 * w.k + 2 * 4 * l1m + 4 * int(w.weights[-1].shape[1])
        out["materialized"] = {"rows_per_s": n / (t[0] * 1e-3), "chunk_rows": chunk, **tstats(t),
                               "roofline": hbm_roofline(bpr, n, t[2], note="non-fused pipeline: materialise T, dense first layer, "
                                                        "second layer; HBM bytes per row as listed in the source; its dense first "
                                                        "layer also stands at the fp32 matrix rate")}
        if "stages" in out:
            out["materialized"]["fused_speedup"] = t[2] / (out["stages"]["fused_join_predict_ms_median"]
                                                          + out["stages"]["project_dims_ms_median"])
    if want("materialized"):
        guarded("materialized", leg_materialized)
    del w, P, Y
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- C1: tiny linear regression (launch-latency sized)
    def leg_c1():
        w1 = WL.c1_tiny_linear(device=dev)
        P1 = [torch.empty((d.shape[0], 1), dtype=torch.float32, device=dev) for d in w1.dims]
        Y1 = torch.empty((w1.n, 1), dtype=torch.float32, device=dev)
        ws1 = torch.empty(lq.lq_workspace_bytes(MAT, w1.k, w1.weights, 16_384), dtype=torch.uint8, device=dev)
        pt = time_call(lambda: lq.lq_project_dims(w1.dims, w1.weights[0], w1.c_f, P=P1), 50, 5)
        ft = time_call(lambda: lq.lq_fused_join_predict(w1.X, w1.fks, P1, w1.weights, None, Y=Y1), 50, 5)
        mt = time_call(lambda: lq.lq_materialized_join_predict(w1.X, w1.dims, w1.fks, w1.weights, None, Y=Y1, ws=ws1), 50, 5)
        gus = graph_time(lambda: lq.lq_fused_join_predict(w1.X, w1.fks, P1, w1.weights, None, Y=Y1), reps=32, iters=20, warmup=3)
        gpus = graph_time(lambda: lq.lq_project_dims(w1.dims, w1.weights[0], w1.c_f, P=P1), reps=32, iters=20, warmup=3)
        gmus = graph_time(lambda: lq.lq_materialized_join_predict(w1.X, w1.dims, w1.fks, w1.weights, None, Y=Y1, ws=ws1),
                          reps=32, iters=20, warmup=3)
        out["fused_c1"] = {"fact_rows": w1.n, "fused_us": ft[0] * 1e3, "fused_us_median": ft[2] * 1e3, "fused_us_min": ft[1] * 1e3,
                           "fused_us_in_a_graph": gus * 1e3, "project_dims_us": pt[2] * 1e3, "project_dims_us_in_a_graph": gpus * 1e3,
                           "materialized_us": mt[2] * 1e3, "materialized_us_in_a_graph": gmus * 1e3, "rows_per_s": w1.n / (gus * 1e-3),
                           "fused_speedup": gmus / (gus + gpus), "fused_speedup_join_stage_alone": gmus / gus,
                           "fused_speedup_at_the_python_callers_pace": mt[2] / (ft[2] + pt[2]),
                           "note": "280 KB of traffic: bound by launch latency; the *_us figures are paced by the Python caller "
                                   "(one call every 15-20 us whatever it launches), the *_in_a_graph ones, rows_per_s and "
                                   "fused_speedup by the GPU (32 calls per graph)"}
        if do_cpu:
            out["fused_c1"]["cpu"] = cpu_predict(w1, w1.n, w1.n)
    if want("c1"):
        guarded("fused_c1", leg_c1)

    # ---------------------------------------------------------------- linear regression at scale (the model of Section 3.2)
    def leg_linear():
        nl = 10_000_000
        cells = {}
        for name, rows, cols in (("c2_star", (1_000, 10_000, 100_000), (32, 32, 32)),
                                 ("dimension_tables_all_in_lds", (1_000, 10_000, 20_000), (32, 32, 32)),
                                 ("four_tables_ssb_sf1_sizes", (2_556, 30_000, 2_000, 200_000), (8, 8, 8, 8))):
            wl = WL.make_predict("linear_" + name, nl, 4, rows, cols, (1,), seed=WL.SEED0 + 800, device=dev, bias=True)
            Pl = lq.lq_project_dims(wl.dims, wl.weights[0], wl.c_f)
            Yl = torch.empty((nl, 1), dtype=torch.float32, device=dev)
            pt = time_call(lambda: lq.lq_project_dims(wl.dims, wl.weights[0], wl.c_f, P=Pl), 10, 2)
            fms = graph_time(lambda: lq.lq_fused_join_predict(wl.X, wl.fks, Pl, wl.weights, wl.biases, Y=Yl))
            chunk = 1 << 21
            wsl = torch.empty(lq.lq_workspace_bytes(MAT, wl.k, wl.weights, chunk), dtype=torch.uint8, device=dev)
            mt = time_call(lambda: lq.lq_materialized_join_predict(wl.X, wl.dims, wl.fks, wl.weights, wl.biases, Y=Yl, ws=wsl), 5, 1)
            bpr = 4 * (4 + len(rows) + 1)
            cells[name] = {"dim_rows": list(rows), "joined_cols": wl.k, "fused_ms_in_a_graph": fms, "project_dims_ms": pt[2],
                           "rows_per_s": nl / (fms * 1e-3), "materialized_ms": mt[2], "fused_speedup": mt[2] / (fms + pt[2]),
                           "roofline": hbm_roofline(bpr, nl, fms)}
            del wl, Pl, Yl, wsl
        out["linear_regression"] = {"fact_rows": nl, "fact_cols": 4, "outputs": 1, "cells": cells}
    if want("linear"):
        guarded("linear_regression", leg_linear)

    # ---------------------------------------------------------------- C3: LA group-by (SSB sf 1 shape)
    def leg_groupby():
        g = WL.c3_groupby(device=dev)
        # rotate over several copies of the fact columns so that repeats are not served from cache
        copies = 6
        cols = [([f.clone() for f in g.fks], [m.clone() for m in g.measures]) for _ in range(copies)]
        ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device=dev)
        sums = torch.empty((1, g.G), dtype=torch.int64, device=dev)
        counts = torch.empty((g.G,), dtype=torch.int64, device=dev)
        it = [0]

        def gb(flags=0):
            fk, me = cols[it[0] % copies]
            it[0] += 1
            lq.lq_masked_groupby_sum(fk, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None, me,
                                     sums=sums, counts=counts, ws=ws, flags=flags)
        t = time_call(gb, 60, 6)
        rt = time_call(lambda: gb(lq.LQ_REUSE_SIDE_TABLES), 60, 6)       # dimension side already encoded in ws
        survivors = int(counts.sum().item())
        # the same calls recorded in a HIP graph (12 per graph, two turns over the copies): no gaps between the launches
        gt = graph_time(gb, reps=2 * copies, iters=20, warmup=3)
        grt = graph_time(lambda: gb(lq.LQ_REUSE_SIDE_TABLES), reps=2 * copies, iters=20, warmup=3)
        # the same query with a selection vector on the fact table itself (one byte per fact row, nine rows in ten kept)
        fact_masks = [(torch.rand(g.n, device=dev) < 0.9).to(torch.uint8) for _ in range(copies)]

        def gb_fact_mask():
            fk, me = cols[it[0] % copies]
            fm = fact_masks[it[0] % copies]
            it[0] += 1
            lq.lq_masked_groupby_sum(fk, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, fm, me,
                                     sums=sums, counts=counts, ws=ws)
        fmt = graph_time(gb_fact_mask, reps=2 * copies, iters=20, warmup=3)
        # floor of this call shape on this machine: one launch that only reads the 96 MB of key columns
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        keys = torch.cat([f.view(torch.uint8) for f in cols[0][0]])
        ft = time_call(lambda: lq.lq_yardstick_read(keys, 1, sink), 30, 5)
        out["groupby_c3"] = {"rows_per_s": g.n / (t[2] * 1e-3), "fact_rows": g.n, "groups": g.G, "surviving_rows": survivors,
                             **tstats(t), **tstats(rt, "reuse_side_tables_"),
                             "ms_in_a_graph": gt, "reuse_side_tables_ms_in_a_graph": grt,
                             "launches_per_call": 3, "read_only_sweep_of_the_key_columns_ms": ft[2],
                             "with_a_fact_mask_ms_in_a_graph": fmt,
                             "roofline": hbm_roofline(20, g.n, t[2], traffic=measured_traffic("groupby_c3"),
                                                      frac_reuse_side_tables=20.0 * g.n / (rt[2] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                                      bytes_per_row_keys_only=16,
                                                      frac_keys_only=16.0 * g.n / (t[2] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                                      note="20 B/row counts the measure column for every row; the scan reads it only "
                                                           "where a lane has a survivor (keys_only = the 16 B/row that are always read)")}
        if do_cpu:
            out["groupby_c3"]["cpu"] = cpu_groupby(g)
        del g, cols
    if want("groupby"):
        guarded("groupby_c3", leg_groupby)

    # ---------------------------------------------------------------- group-by with more groups than LDS accumulators
    def leg_groupby_many():
        nm = 6_000_000
        cells = {}
        for name, rows, card, sel in (("three_attributes_25x25x250_selective", (2_556, 30_000, 2_000, 200_000), (25, 25, 250, 1), (None, 0.2, None, 0.12)),
                                      ("three_attributes_25x25x250_all_rows", (2_556, 30_000, 2_000, 200_000), (25, 25, 250, 1), (None, None, None, 1.0)),
                                      ("two_attributes_250x250_selective", (2_556, 30_000, 2_000, 200_000), (250, 250, 1, 1), (None, None, 0.2, 0.12)),
                                      # year x brand with a filter on the supplier side: a grouping attribute of 1,000 values
                                      ("year_x_1000_brands_one_supplier_region", (2_556, 30_000, 2_000, 200_000), (7, 1, 1, 1_000), (None, 1.0, 0.2, None))):
            gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 970)
            fks = [torch.randint(0, r, (nm,), generator=gen, device=dev, dtype=torch.int32) for r in rows]
            codes = [torch.randint(0, c, (r,), generator=gen, device=dev, dtype=torch.int32) if c > 1 else None for r, c in zip(rows, card)]
            masks = [None if sel is None or sel[k] is None else (torch.rand(rows[k], generator=gen, device=dev) < sel[k]).to(torch.uint8)
                     for k in range(len(rows))]
            meas = [torch.randint(1, 100_001, (nm,), generator=gen, device=dev, dtype=torch.int32)]
            G = math.prod(card)
            small = lq.lq_groupby_workspace_bytes(rows, card, 1)
            big = lq.lq_groupby_bucket_workspace_bytes(nm, rows, card, 1)
            ws = torch.empty(max(small, big), dtype=torch.uint8, device=dev)
            sums = torch.empty((1, G), dtype=torch.int64, device=dev)
            counts = torch.empty((G,), dtype=torch.int64, device=dev)
            t = time_call(lambda: lq.lq_masked_groupby_sum(fks, rows, masks, codes, card, None, meas, sums=sums, counts=counts, ws=ws), 20, 3)
            at = time_call(lambda: lq.lq_masked_groupby_sum(fks, rows, masks, codes, card, None, meas, sums=sums, counts=counts,
                                                            ws=ws[:small]), 20, 3)
            cells[name] = {"groups": G, "surviving_rows": int(counts.sum().item()), "rows_per_s": nm / (t[2] * 1e-3), **tstats(t),
                           "through_atomics_ms": at[2], "workspace_MB": max(small, big) / 1e6, "workspace_for_atomics_MB": small / 1e6,
                           "roofline": hbm_roofline(20, nm, t[2])}
        out["groupby_many_groups"] = {"fact_rows": nm, "cells": cells,
                                      "note": "above 8,192 accumulators: with the large workspace survivors are sorted into buckets of "
                                              "neighbouring groups and each bucket is added up in LDS by the workgroup that owns it "
                                              "(ms); with the small one the output arrays accumulate through device-wide 64-bit atomics, "
                                              "about 2.3e10 per second on this GPU (through_atomics_ms)"}
    if want("groupby_many"):
        guarded("groupby_many_groups", leg_groupby_many)

    # ---------------------------------------------------------------- C4: skewed linear model (HBM-bound)
    def leg_c4():
        n4 = 100_000_000
        w4 = WL.c4_skewed(device=dev, n=n4)
        P4 = [torch.empty((d.shape[0], 4), dtype=torch.float32, device=dev) for d in w4.dims]
        Y4 = torch.empty((n4, 4), dtype=torch.float32, device=dev)
        pt = time_call(lambda: lq.lq_project_dims(w4.dims, w4.weights[0], w4.c_f, P=P4), 10, 2)
        t = time_call(lambda: lq.lq_fused_join_predict(w4.X, w4.fks, P4, w4.weights, None, Y=Y4), 20, 3)
        # what the two halves of this kernel cost alone on this machine: the stream (read X, write Y: a copy of the same
        # bytes) and the gathers (the real key columns, 16-byte rows, nothing else)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        st = time_call(lambda: lq.lq_yardstick_stream(w4.X, 1, Y4, sink), 10, 2)
        gt = time_call(lambda: (lq.lq_yardstick_gather(P4[0], 16, n4, sink, keys=w4.fks[0]),
                                lq.lq_yardstick_gather(P4[1], 16, n4, sink, keys=w4.fks[1])), 10, 2)
        m4 = 1 << 23                                  # non-fused pipeline on a slice: T of all rows is 106 GB
        ws4 = torch.empty(lq.lq_workspace_bytes(MAT, w4.k, w4.weights, 1 << 21), dtype=torch.uint8, device=dev)
        Ym4 = torch.empty((m4, 4), dtype=torch.float32, device=dev)
        mt = time_call(lambda: lq.lq_materialized_join_predict(w4.X[:m4], w4.dims, [f[:m4] for f in w4.fks],
                                                               w4.weights, None, Y=Ym4, ws=ws4), 5, 1)
        out["fused_c4"] = {"rows_per_s": n4 / (t[2] * 1e-3), **tstats(t), "project_dims_ms": pt[2], "fact_rows": n4,
                           "materialized_rows_per_s": m4 / (mt[2] * 1e-3), "materialized_slice_rows": m4,
                           "fused_speedup": (mt[2] / m4) / ((t[2] + pt[2]) / n4),
                           "roofline": hbm_roofline(56, n4, t[2], traffic=measured_traffic("fused_c4"),
                                                    stream_only_ms=st[2], gathers_only_ms=gt[2],
                                                    frac_of_stream_plus_gathers=(st[2] + gt[2]) / t[2],
                                                    frac_of_the_slower_half=max(st[2], gt[2]) / t[2],
                                                    note="stream_only = one launch that reads X and overwrites Y (48 B/row of the 56); "
                                                         "gathers_only = the 2e8 random 16-byte reads through the real key columns "
                                                         "(8 B/row of keys streamed); the kernel does both at once"),
                           "project_dims_GBps": 2 * 1_000_000 * 128 * 4 / (pt[2] * 1e-3) / 1e9}
        if do_cpu:
            out["fused_c4"]["cpu"] = cpu_predict(w4, 1 << 24, 1 << 21)
    if want("c4"):
        guarded("fused_c4", leg_c4)

    # ---------------------------------------------------------------- C5: wide bf16 MLP (cache-gather bound)
    def leg_c5():
        n5 = 50_000_000
        w5 = WL.c5_wide_bf16(device=dev, n=n5)
        P5 = [torch.empty((d.shape[0], 256), dtype=torch.bfloat16, device=dev) for d in w5.dims]
        Y5 = torch.empty((n5, 16), dtype=torch.bfloat16, device=dev)
        pt = time_call(lambda: lq.lq_project_dims(w5.dims, w5.weights[0], 0, P=P5), 10, 2)
        t = time_call(lambda: lq.lq_fused_join_predict(None, w5.fks, P5, w5.weights, None, Y=Y5), 10, 2)
        m5 = 1 << 22                                  # non-fused pipeline on a slice: T of all rows is 102 GB
        ws5 = torch.empty(lq.lq_workspace_bytes(MAT, w5.k, w5.weights, 1 << 20), dtype=torch.uint8, device=dev)
        fk5 = [f[:m5] for f in w5.fks]
        Ym5 = torch.empty((m5, 16), dtype=torch.bfloat16, device=dev)
        mt = time_call(lambda: lq.lq_materialized_join_predict(None, w5.dims, fk5, w5.weights, None, Y=Ym5, ws=ws5), 5, 1)
        ggbps = 2048.0 * n5 / (t[2] * 1e-3) / 1e9
        yg = yard.get("gather_512B_rows_of_20.5MB_GBps")
        out["fused_c5"] = {"rows_per_s": n5 / (t[2] * 1e-3), **tstats(t), "project_dims_ms": pt[2], "fact_rows": n5,
                           "dtype": "bf16", "gather_GBps": ggbps, "gather_yardstick_GBps": yg,
                           "gather_frac_of_yardstick": (ggbps / yg) if yg else None,
                           "hbm_GBps_algorithmic": 48.0 * n5 / (t[2] * 1e-3) / 1e9,
                           "materialized_rows_per_s": m5 / (mt[2] * 1e-3), "materialized_slice_rows": m5,
                           "fused_speedup": (mt[2] / m5) / ((t[2] + pt[2]) / n5)}
        if do_cpu:
            out["fused_c5"]["cpu"] = cpu_predict(w5, 1 << 16, 1 << 13)
    if want("c5"):
        guarded("fused_c5", leg_c5)

    # ---------------------------------------------------------------- deeper models (later layers on the matrix cores)
    def leg_deep():
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
            t = time_call(lambda: lq.lq_fused_join_predict(wd.X, wd.fks, Pd, wd.weights, None, Y=Yd), 10, 2)
            wsd = torch.empty(lq.lq_workspace_bytes(MAT, wd.k, wd.weights, 1 << 20), dtype=torch.uint8, device=dev)
            mt = time_call(lambda: lq.lq_materialized_join_predict(wd.X, wd.dims, wd.fks, wd.weights, None, Y=Yd, ws=wsd), 5, 1)
            later_flop = 2.0 * sum(a * b for a, b in zip(layers[:-1], layers[1:])) * nd
            cells[name] = {"fused_ms": round(t[2], 4), "fused_ms_min": round(t[1], 4), "rows_per_s": nd / (t[2] * 1e-3),
                           "later_layers_TFLOPs": later_flop / (t[2] * 1e-3) / 1e12,
                           # fp32 cells: time of the matrix instructions alone (widths padded to 16, fact columns to 4) at
                           # the measured matrix rate, over the kernel's time; the vector work in between is not hidden
                           "matrix_pipe_busy_frac": (None if dt != torch.float32 or not yard.get("fp32_matrix_TFLOPs") else
                                                     2.0 * nd * (sum(-(-a // 16) * 16 * -(-b // 16) * 16 for a, b in zip(layers[:-1], layers[1:])
                                                                     if b > 1) + -(-c_f // 4) * 4 * -(-layers[0] // 16) * 16)
                                                     / (t[2] * 1e-3) / (yard["fp32_matrix_TFLOPs"] * 1e12)),
                           "gather_GBps": len(rows) * layers[0] * wd.dims[0].element_size() * nd / (t[2] * 1e-3) / 1e9,
                           "materialized_ms": round(mt[2], 3), "fused_speedup": mt[2] / t[2]}
            del wd, Pd, Yd, wsd
        out["deeper_models"] = {"fact_rows": nd, "cells": cells}
    if want("deep"):
        guarded("deeper_models", leg_deep)

    # ---------------------------------------------------------------- wide models (layered form: linear join stage + dense layers)
    def leg_wide_models():
        nw = 1_000_000
        cells = {}
        for name, dt, layers in (("f32_1024_1024", torch.float32, (1024, 1024)), ("f32_512_64_1", torch.float32, (512, 64, 1)),
                                 ("f32_2048_256", torch.float32, (2048, 256)), ("bf16_1024_64_1", torch.bfloat16, (1024, 64, 1))):
            ww = WL.make_predict(name, nw, 4, (1_000, 10_000, 100_000), (32, 32, 32), layers, seed=WL.SEED0 + 960, dtype=dt, device=dev,
                                 w_sigma=[0.05] * len(layers))
            Pw = lq.lq_project_dims(ww.dims, ww.weights[0], 4, p_dtype=dt)
            Yw = torch.empty((nw, layers[-1]), dtype=dt, device=dev)
            ws_l = torch.empty(lq.lq_workspace_bytes(lq.binding.LQ_CALL_FUSED, ww.k, ww.weights, 1 << 17), dtype=torch.uint8, device=dev)
            t = time_call(lambda: lq.lq_fused_join_predict(ww.X, ww.fks, Pw, ww.weights, None, Y=Yw, ws=ws_l), 5, 1)
            wsm = torch.empty(lq.lq_workspace_bytes(MAT, ww.k, ww.weights, 1 << 17), dtype=torch.uint8, device=dev)
            mt = time_call(lambda: lq.lq_materialized_join_predict(ww.X, ww.dims, ww.fks, ww.weights, None, Y=Yw, ws=wsm), 3, 1)
            later = 2.0 * sum(a * b for a, b in zip(layers[:-1], layers[1:])) * nw
            cells[name] = {"fused_ms": round(t[2], 3), "rows_per_s": nw / (t[2] * 1e-3), "later_layers_TFLOPs": later / (t[2] * 1e-3) / 1e12,
                           "materialized_ms": round(mt[2], 3), "fused_speedup": mt[2] / t[2], "workspace_MB": ws_l.numel() / 1e6}
            del ww, Pw, Yw, ws_l, wsm
        out["wide_models"] = {"fact_rows": nw, "cells": cells,
                              "note": "models no fused kernel takes: the join stage as a linear operator with the ReLU in its store, "
                                      "later layers as dense products, in chunks of 131,072 rows"}
    if want("wide_models"):
        guarded("wide_models", leg_wide_models)

    # ---------------------------------------------------------------- group-by at 16x the fact rows
    def leg_groupby16():
        g = WL.c3_groupby(device=dev, n=96_000_000, dim_rows=(2_556, 480_000, 32_000, 1_000_000))
        ws = torch.empty(lq.lq_groupby_workspace_bytes(g.dim_rows, g.group_card, 1), dtype=torch.uint8, device=dev)
        sums = torch.empty((1, g.G), dtype=torch.int64, device=dev)
        counts = torch.empty((g.G,), dtype=torch.int64, device=dev)
        t = time_call(lambda: lq.lq_masked_groupby_sum(g.fks, g.dim_rows, g.dim_mask, g.dim_code, g.group_card, None,
                                                       g.measures, sums=sums, counts=counts, ws=ws), 20, 3)
        out["groupby_sf16_shape"] = {"rows_per_s": g.n / (t[2] * 1e-3), **tstats(t), "fact_rows": g.n, "dim_rows": list(g.dim_rows),
                                     "roofline": hbm_roofline(20, g.n, t[2])}
        del g
    if want("groupby16"):
        guarded("groupby_sf16_shape", leg_groupby16)

    # ---------------------------------------------------------------- decision tree (setting 1, sf 8)
    def leg_tree():
        nt = 4_800_000
        wt = WL.make_predict("tree_s1_sf8", nt, 0, (80_000, 16_000, 2_555), (43, 43, 42), (1,),
                             seed=WL.SEED0 + 700, device=dev)
        tree = WL.make_tree(128, 64, WL.SEED0 + 701)
        tf, tt, tH = tree.feature.to(dev), tree.threshold.to(dev), tree.H.to(dev)
        tables, target = lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH)
        pms = time_call(lambda: lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH), 5, 1)[2]
        t = time_call(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH), 20, 3)
        ms = t[2]
        mms = time_call(lambda: lq.lq_materialized_join_tree(None, wt.dims, wt.fks, tf, tt, tH, chunk_rows=1 << 20), 5, 1)[2]
        # leaf masks: the same tables compressed to one bit per leaf, AND instead of sum-and-compare
        masks = lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH)
        cms = time_call(lambda: lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH), 5, 1)[2]
        kms = time_call(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH), 20, 3)[2]
        gms = graph_time(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH))
        kgms = graph_time(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH))
        out["fused_tree"] = {"rows_per_s": nt / (ms * 1e-3), **tstats(t), "project_ms": pms, "fact_rows": nt,
                             "leaves": 64, "nodes": 63, "joined_cols": 128,
                             "materialized_rows_per_s": nt / (mms * 1e-3),
                             "fused_speedup": mms / (ms + pms),
                             "roofline": hbm_roofline(16, nt, ms, gather_GBps=192.0 * nt / (ms * 1e-3) / 1e9),
                             "ms_in_a_graph": gms,
                             "leaf_masks": {"rows_per_s": nt / (kgms * 1e-3), "ms": kms, "ms_in_a_graph": kgms,
                                            "compress_ms": cms,
                                            "fused_speedup": mms / (kms + pms + cms),
                                            "roofline": hbm_roofline(16, nt, kgms)}}
        del wt, tables, masks
        # the same tree size with 8 of the 128 joined columns in the fact table itself: their nodes are
        # evaluated per fact row in the join stage
        wf = WL.make_predict("tree_s1_sf8_fact", nt, 8, (80_000, 16_000, 2_555), (40, 40, 40), (1,),
                             seed=WL.SEED0 + 702, device=dev)
        tables, target = lq.lq_tree_project_dims(wf.dims, 8, tf, tt, tH)
        masks = lq.lq_tree_compress_tables(wf.dims, tables, tf, tt, tH, c_f=8)
        fmask = lq.lq_tree_fact_masks(8, tf, tt, tH)
        fcnt = int(fmask[:4].view(torch.int32).item())
        fms = time_call(lambda: lq.lq_fused_join_tree(wf.X, wf.fks, tables, target, tf, tt, tH), 5, 1)[2]
        fkms = graph_time(lambda: lq.lq_fused_join_tree_masks(wf.fks, masks, tf, tt, tH, X=wf.X, fact_masks=fmask))
        fmms = time_call(lambda: lq.lq_materialized_join_tree(wf.X, wf.dims, wf.fks, tf, tt, tH, chunk_rows=1 << 20), 5, 1)[2]
        out["fused_tree"]["with_fact_columns"] = {
            "fact_cols": 8, "nodes_on_fact_cols": fcnt, "byte_tables_ms": fms, "leaf_masks_ms_in_a_graph": fkms,
            "materialized_ms": fmms, "fused_speedup_join_stage": fmms / fkms,
            "roofline": hbm_roofline(48, nt, fkms)}
        del wf, tables, masks, fmask
    if want("tree"):
        guarded("fused_tree", leg_tree)

    # ---------------------------------------------------------------- trees of growing size
    # cardinality settings 1 (large dimension tables, sf 4) and 2 (small ones), leaves 8 .. 2,048:
    # where the pre-fusion stage starts to dominate (Section 4.4, the tree experiments)
    def leg_treesweep():
        cells = {}
        for setting, nt, rows in (("setting1_sf4", 2_400_000, (40_000, 8_000, 2_555)),
                                  ("setting2", 2_400_000, (1_000, 500, 2_555))):
            wt = WL.make_predict("tree_sweep", nt, 0, rows, (43, 43, 42), (1,), seed=WL.SEED0 + 720, device=dev)
            for leaves in (8, 64, 256, 1024, 2048):
                tree = WL.make_tree(128, leaves, WL.SEED0 + 721 + leaves)
                tf, tt, tH = tree.feature.to(dev), tree.threshold.to(dev), tree.H.to(dev)
                tables, target = lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH)
                pms = time_call(lambda: lq.lq_tree_project_dims(wt.dims, 0, tf, tt, tH), 3, 1)[2]
                mms = time_call(lambda: lq.lq_materialized_join_tree(None, wt.dims, wt.fks, tf, tt, tH,
                                                                     chunk_rows=1 << 19), 2 if leaves >= 1024 else 3, 1)[2]
                masks = lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH)
                cms = time_call(lambda: lq.lq_tree_compress_tables(wt.dims, tables, tf, tt, tH), 3, 1)[2]
                gms = graph_time(lambda: lq.lq_fused_join_tree(None, wt.fks, tables, target, tf, tt, tH), 8, 5, 1)
                kgms = graph_time(lambda: lq.lq_fused_join_tree_masks(wt.fks, masks, tf, tt, tH), 8, 5, 1)
                cells[f"{setting}_l{leaves}"] = {"fused_ms_in_a_graph": round(gms, 4), "prefusion_ms": round(pms, 4),
                                                 "materialized_ms": round(mms, 3),
                                                 "speedup_join_stage": round(mms / gms, 1),
                                                 "speedup_with_prefusion": round(mms / (gms + pms), 1),
                                                 "masks_fused_ms_in_a_graph": round(kgms, 4),
                                                 "masks_compress_ms": round(cms, 4),
                                                 "masks_speedup_join_stage": round(mms / kgms, 1),
                                                 "masks_speedup_with_prefusion": round(mms / (kgms + pms + cms), 1)}
                del tables, masks
            del wt
            torch.cuda.empty_cache()
        out["tree_sweep"] = {"fact_rows": 2_400_000, "joined_cols": 128, "cells": cells}
    if want("treesweep"):
        guarded("tree_sweep", leg_treesweep)

    # ---------------------------------------------------------------- key -> row mapping (SSB sf1 shape)
    def leg_keymap():
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
            bms = time_call(lambda: lq.lq_keymap_build(keys_S), 5, 1)[2]
            lms = time_call(lambda: lq.lq_keymap_lookup(table, fact, fk=fk), 20, 3)[2]
            res[str(r)] = {"build_ms": bms, "lookup_ms": lms, "lookup_GBps": 8.0 * nk / (lms * 1e-3) / 1e9}
            tot_ms += lms
            # surrogate keys 1..r in shuffled row order: the dense range makes the map a direct array
            keys_D = (torch.randperm(r, generator=gen, device=dev) + 1).to(torch.int32)
            fact_D = keys_D[torch.randint(0, r, (nk,), generator=gen, device=dev)]
            table_D = lq.lq_keymap_build(keys_D)
            dbms = time_call(lambda: lq.lq_keymap_build(keys_D), 5, 1)[2]
            dlms = time_call(lambda: lq.lq_keymap_lookup(table_D, fact_D, fk=fk), 20, 3)[2]
            res[str(r)].update({"dense_build_ms": dbms, "dense_lookup_ms": dlms,
                                "dense_lookup_GBps": 8.0 * nk / (dlms * 1e-3) / 1e9})
            tot_dense += dlms
        out["keymap_ssb_sf1"] = {"fact_rows": nk, "rows_per_s_all_4_columns": nk / (tot_ms * 1e-3),
                                 "dense_keys_rows_per_s_all_4_columns": nk / (tot_dense * 1e-3), "per_dimension": res,
                                 "roofline": hbm_roofline(8, 4 * nk, tot_ms)}
        gy = yard.get("gather_16B_rows_of_2MB_Grows_per_s")
        if gy:
            # a hashed lookup is at least one random 8-byte read of a table that sits in L2: the rate of the bare gather
            # yardstick (16-byte rows of a 2 MB table) is its roof, the 8 bytes per key streamed in and out are not
            big = res["200000"]["lookup_ms"]
            out["keymap_ssb_sf1"]["hashed_lookups_frac_of_gather_yardstick"] = (nk / (big * 1e-3) / 1e9) / gy
            out["keymap_ssb_sf1"]["note"] = ("hashed_lookups_frac_of_gather_yardstick: keys per second into the 200,000-key map "
                                             "(3.2 MB of slots at load factor 1/2, 1.5 probes on average) over random 16-byte "
                                             "reads per second from a 2 MB table")
    if want("keymap"):
        guarded("keymap_ssb_sf1", leg_keymap)

    # ---------------------------------------------------------------- wider aggregate (1 join, fact predicates, SUM(a*b))
    def leg_agg():
        na = 6_000_000
        gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 950)
        ri = lambda lo, hi: torch.randint(lo, hi, (na,), generator=gen, device=dev, dtype=torch.int32)
        fk = ri(0, 2_556)
        price, disc, qty = ri(1, 100_001), ri(0, 11), ri(1, 51)
        dmask = (torch.arange(2_556, device=dev) % 7 == 3).to(torch.uint8)
        call = lambda: lq.lq_groupby_agg([fk], [2_556], [dmask], [None], [1], [(disc, 1, 3), (qty, 1, 24)],
                                         [("mul", price, disc)], want=("sum", "count"))
        t = time_call(call, 30, 3)
        out["agg_one_join"] = {"rows_per_s": na / (t[2] * 1e-3), **tstats(t), "fact_rows": na, "roofline": hbm_roofline(16, na, t[2])}
    if want("agg"):
        guarded("agg_one_join", leg_agg)

    # ---------------------------------------------------------------- group discovery + ORDER BY (query set-up / tail)
    def leg_domain():
        gen = torch.Generator(device=dev); gen.manual_seed(WL.SEED0 + 960)
        rd = 1_400_000                                                       # part dimension at sf 16
        a5 = torch.randint(0, 5, (rd,), generator=gen, device=dev, dtype=torch.int32) * 11 + 3
        b25 = a5 * 5 + torch.randint(0, 5, (rd,), generator=gen, device=dev, dtype=torch.int32)
        dms = time_call(lambda: lq.lq_group_domain([a5, b25]), 10, 2)[2]     # includes its one host wait
        Gd = 7 * 25
        cnt = torch.randint(0, 1000, (Gd,), generator=gen, device=dev, dtype=torch.int64)
        sm = torch.randint(0, 1 << 40, (1, Gd), generator=gen, device=dev, dtype=torch.int64)
        o_buf = torch.empty(8192, dtype=torch.int32, device=dev)
        n_buf = torch.empty(1, dtype=torch.int32, device=dev)
        oms = time_call(lambda: lq.lq_order_groups([7, 25], sm, cnt, [(0, 0, False), (1, 0, True)], order=o_buf, n_out=n_buf), 20, 3)[2]
        cnt8 = torch.randint(0, 3, (8192,), generator=gen, device=dev, dtype=torch.int64)
        sm8 = torch.randint(0, 1 << 40, (1, 8192), generator=gen, device=dev, dtype=torch.int64)
        oms8 = time_call(lambda: lq.lq_order_groups([64, 128], sm8, cnt8, [(1, 0, True)], order=o_buf, n_out=n_buf), 20, 3)[2]
        out["group_domain_and_order"] = {"group_domain_ms": dms, "dim_rows": rd, "columns": 2, "groups": 25,
                                         "order_175_groups_ms": oms, "order_8192_groups_ms": oms8}
    if want("domain"):
        guarded("group_domain_and_order", leg_domain)

    # ---------------------------------------------------------------- k x l sweep (setting 1, sf 4, linear operator)
    def leg_sweep():
        ns = 2_400_000
        rows_s = (60_000, 8_000, 2_555)
        split = {16: (8, 4, 4), 32: (12, 12, 8), 64: (24, 20, 20), 128: (44, 44, 40)}
        sweep = {}
        ws_s = None
        agree = 0
        for k_in, cols in split.items():
            for l_out in (2, 4, 8, 16, 32, 64, 128):
                wk = WL.make_predict("sweep", ns, 0, rows_s, cols, (l_out,), seed=WL.SEED0 + 1000 + k_in, device=dev)
                Pk = lq.lq_project_dims(wk.dims, wk.weights[0], 0)
                Yk = torch.empty((ns, l_out), dtype=torch.float32, device=dev)
                fms = time_call(lambda: lq.lq_fused_join_predict(None, wk.fks, Pk, wk.weights, None, Y=Yk), 5, 1)[2]
                pms = time_call(lambda: lq.lq_project_dims(wk.dims, wk.weights[0], 0, P=Pk), 5, 1)[2]
                need = lq.lq_workspace_bytes(MAT, k_in, wk.weights, 1 << 21)
                if ws_s is None or ws_s.numel() < need:
                    ws_s = torch.empty(need, dtype=torch.uint8, device=dev)
                mms = time_call(lambda: lq.lq_materialized_join_predict(None, wk.dims, wk.fks, wk.weights, None, Y=Yk, ws=ws_s), 5, 1)[2]
                adv = lq.lq_fusion_advice(ns, 0, list(zip(rows_s, cols)), [l_out], queries_per_update=1.0)
                agree += int(adv["fuse"] == int(mms > fms + pms))
                sweep[f"k{k_in}_l{l_out}"] = {"fused_ms": round(fms, 4), "prefusion_ms": round(pms, 4),
                                              "materialized_ms": round(mms, 4), "speedup": round(mms / fms, 2),
                                              "k_over_l": k_in / l_out, "advice_fuse": adv["fuse"]}
        out["sweep_setting1_sf4"] = {"fact_rows": ns, "dim_rows": list(rows_s), "cells": sweep,
                                     "advice_agrees_with_measurement_in_cells": agree, "cells_total": len(sweep)}
    if want("sweep"):
        guarded("sweep_setting1_sf4", leg_sweep)

    # ---------------------------------------------------------------- cardinality setting 2: small tables, wide operators
    # (Table 4 / Table 5: fact sf * 3,000 rows, part 2,000 * floor(1 + log2 sf), supplier sf * 2,000, date 2,555 rows;
    # k = 2^8 .. 2^11, l up to k).  Pre-fusion and join stage are reported separately: the regime of Q6,
    # where the pre-fusion stage dominates.  The join stage is timed at the GPU's pace (calls recorded in a graph).
    def leg_setting2():
        cells = {}
        for sf in (2, 4):
            nf = sf * 3_000
            rows2 = (2_000 * int(1 + math.log2(sf)), sf * 2_000, 2_555)
            for k_in, l_out in ((256, 256), (256, 1024), (256, 2048), (1024, 512), (1024, 1024), (2048, 512), (2048, 2048)):
                base = k_in // 3
                cols = tuple(base + (1 if i < k_in - 3 * base else 0) for i in range(3))
                wk = WL.make_predict("setting2", nf, 0, rows2, cols, (l_out,), seed=WL.SEED0 + 1100 + k_in, device=dev,
                                     w_sigma=[1.0 / math.sqrt(k_in)])
                Pk = lq.lq_project_dims(wk.dims, wk.weights[0], 0)
                Yk = torch.empty((nf, l_out), dtype=torch.float32, device=dev)
                ws2 = torch.empty(lq.lq_workspace_bytes(MAT, k_in, wk.weights, nf), dtype=torch.uint8, device=dev)
                jms = graph_time(lambda: lq.lq_fused_join_predict(None, wk.fks, Pk, wk.weights, None, Y=Yk), 8, 5, 1)
                pms = graph_time(lambda: lq.lq_project_dims(wk.dims, wk.weights[0], 0, P=Pk), 4, 5, 1)
                mms = graph_time(lambda: lq.lq_materialized_join_predict(None, wk.dims, wk.fks, wk.weights, None, Y=Yk, ws=ws2), 4, 5, 1)
                moved = nf * (3 * l_out * 4 + l_out * 4 + 12)          # gathered rows + output + keys
                pflop = 2.0 * sum(r * c for r, c in zip(rows2, cols)) * l_out
                cells[f"sf{sf}_k{k_in}_l{l_out}"] = {
                    "join_stage_ms": round(jms, 4), "prefusion_ms": round(pms, 4), "materialized_ms": round(mms, 4),
                    "prefusion_share": round(pms / (pms + jms), 3),
                    "speedup_join_stage": round(mms / jms, 1), "speedup_with_prefusion": round(mms / (jms + pms), 2),
                    "join_stage_GBps_moved": round(moved / (jms * 1e-3) / 1e9, 1),
                    "prefusion_TFLOPs": round(pflop / (pms * 1e-3) / 1e12, 1),
                    "projected_tables_MB": round(sum(rows2) * l_out * 4 / 1e6, 1)}
                del wk, Pk, Yk, ws2
        out["setting2_wide_operators"] = {"cells": cells,
                                          "note": "fp32 linear operator, no fact columns; all three calls at the GPU's pace (recorded in "
                                                  "HIP graphs): at 6,000 / 12,000 fact rows an eager call is paced by its Python caller"}
    if want("setting2"):
        guarded("setting2_wide_operators", leg_setting2)

    # ---------------------------------------------------------------- group-by over scale factors 1..16
    # (the table cardinalities grow as in Section 4.1; rows/s over sf is the scaling curve)
    def leg_sfsweep():
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
            t = time_call(gb, 10, 3)
            cells[f"sf{sf}"] = {"fact_rows": g.n, "dim_rows": list(rows_sf), "ms": round(t[2], 4), "ms_min": round(t[1], 4),
                                "rows_per_s": g.n / (t[2] * 1e-3), "GBps": 20.0 * g.n / (t[2] * 1e-3) / 1e9}
            del g, cols, ws
            torch.cuda.empty_cache()
        out["groupby_sf_sweep"] = cells
    if want("sfsweep"):
        guarded("groupby_sf_sweep", leg_sfsweep)

    # ---------------------------------------------------------------- the named configurations in a few numbers (last key)
    def pick(cell, *path):
        v = out.get(cell)
        for p in path:
            v = v.get(p) if isinstance(v, dict) else None
        return v

    if args.only == "":
        r3 = lambda v: None if v is None else float(f"{v:.4g}")
        out["summary"] = {
            "c1": {"us_in_a_graph": r3(pick("fused_c1", "fused_us_in_a_graph")), "rows_per_s": r3(pick("fused_c1", "rows_per_s")),
                   "speedup": r3(pick("fused_c1", "fused_speedup"))},
            "c2": {"ms_step": r3(out.get("ms_per_step")), "rows_per_s": r3(out.get("value")), "hbm_frac": r3(pick("roofline", "frac")),
                   "gather_frac_of_yardstick": r3(pick("roofline", "gather_frac_of_yardstick")),
                   "speedup": r3(pick("materialized", "fused_speedup")), "cpu_rows_per_s": r3(pick("cpu_baseline", "value"))},
            "c3": {"ms": r3(pick("groupby_c3", "ms_median")), "rows_per_s": r3(pick("groupby_c3", "rows_per_s")),
                   "hbm_frac": r3(pick("groupby_c3", "roofline", "frac")),
                   "hbm_frac_sf16_shape": r3(pick("groupby_sf16_shape", "roofline", "frac")),
                   "cpu_rows_per_s": r3(pick("groupby_c3", "cpu", "all_threads", "rows_per_s"))},
            "c4": {"ms": r3(pick("fused_c4", "ms_median")), "rows_per_s": r3(pick("fused_c4", "rows_per_s")),
                   "hbm_frac": r3(pick("fused_c4", "roofline", "frac")),
                   "frac_of_stream_plus_gathers": r3(pick("fused_c4", "roofline", "frac_of_stream_plus_gathers")),
                   "speedup": r3(pick("fused_c4", "fused_speedup")),
                   "cpu_rows_per_s": r3(pick("fused_c4", "cpu", "all_threads", "rows_per_s"))},
            "c5": {"ms": r3(pick("fused_c5", "ms_median")), "rows_per_s": r3(pick("fused_c5", "rows_per_s")),
                   "gather_frac_of_yardstick": r3(pick("fused_c5", "gather_frac_of_yardstick")),
                   "speedup": r3(pick("fused_c5", "fused_speedup")),
                   "cpu_rows_per_s": r3(pick("fused_c5", "cpu", "all_threads", "rows_per_s"))},
            "host_threads_used_by_the_oracle": cpu_threads() if do_cpu else None,
        }

    # the contract's keys and the per-configuration summary first (a reader that keeps only the head of the line still
    # has every headline figure), the detailed cells after them
    head = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
            "dtype", "data", "config", "roofline", "cpu_baseline", "summary")
    ordered = {k: out[k] for k in head if k in out}
    ordered.update({k: v for k, v in out.items() if k not in ordered})
    print(json.dumps(ordered))


if __name__ == "__main__":
    main()
