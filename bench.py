#!/usr/bin/env python3
"""Benchmark of the retrieval hot path on one MI355X.

Workload of the timed step: the 1 M x 768 fp16 clustered corpus of configurations 1 and 2 of the
workload table, all inputs resident in HBM before the timed region.  One step = one pass of the
whole hot path over one batch of the configuration's own queries:

    flat exact search, B = 16    (streaming kernel, HBM bound)
    flat exact search, B = 512   (matrix-core kernel, MFMA bound)
    graph search, B = 512, at the cheapest search range ef that reaches recall@3 >= 0.95 against
        exact search (the operating point the metric names).  The configuration's literal graph
        (cluster-restricted 32-NN, one shared entry node) has no edges between clusters and cannot
        reach it at any ef, so this leg runs on the same corpus and the same queries with a
        navigable form of the same graph (half of every row replaced by reverse edges, still 32
        slots) and a per-query entry node from an exact search over one representative per
        cluster; that coarse search is part of the leg.  The literal graph is reported next to it.

`value` = queries/s of the graph leg at that operating point (B / leg time, coarse entry search
included).  The flat legs are reported as fractions of the HBM / MFMA peaks beside it.  Further
legs, timed in the same run outside the step: configuration 3 (21 M rows, flat B = 1 / 16 / 256)
and configuration 4 (10 M rows, graph ef = 32 / 64 / 128 at B = 256).  The CPU oracle is timed in
the same run on the host cores on a bounded sample, as a reported baseline.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "queries/sec at recall@3≥0.95 (graph) and flat-scan HBM GB/s / MFMA % of peak"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA
K = 3
RECALL_TARGET = 0.95
B_SMALL, B_LARGE = 16, 512
EF_CANDIDATES = (1024, 2048, 4096, 6144, 8192, 12288, 16384)
TRAFFIC_FILE = "profiles/hbm_traffic_bench_step.md"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic() -> dict:
    """HBM bytes per launch of each main kernel from the committed counter profile of this command
    (rows `| kernel | fetch bytes | write bytes | total | ...`).  Counter passes are separate profiler
    runs, so the figure is not measured in this run; a missing file gives {}."""
    out = {}
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_FILE)):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 4 and cells[0].endswith("_kernel"):
                try:
                    out[cells[0]] = float(cells[3])
                except ValueError:
                    pass
    except OSError:
        pass
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--ef", type=int, default=0, help="search range of the graph leg (0: found by the recall sweep)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the untimed per-B / per-ef report")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline and the oracle counters")
    ap.add_argument("--no-large", action="store_true", help="skip the configuration 3 and 4 legs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2505_12065_amd as ann
    from paper_2505_12065_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t_start = time.time()

    def timed(fn, n=10, w=2):
        for _ in range(w):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def recall3(ids, ref):
        got = ids.cpu().numpy() if hasattr(ids, "cpu") else ids
        return float(np.mean([len(set(got[b].tolist()) & set(ref[b].tolist())) / K for b in range(got.shape[0])]))

    # ---- inputs (untimed): corpus, queries, graphs, entries; all device resident -------------
    corpus = synth.workload_corpus(1, device=dev)
    x = corpus.x
    N, d = x.shape
    q_all = synth.make_queries(corpus, B_LARGE)                 # the configuration's queries: noise std 0.05
    q_small = q_all[:B_SMALL].contiguous()
    graph = synth.knn_graph_cluster_restricted(corpus, 32, 8)    # the configuration's graph
    R = graph.shape[1]
    entry = synth.mean_entry(x)                                  # the configuration's entry node
    graph_nav = synth.with_reverse_edges(graph, x)               # navigable form, same degree
    reps = synth.cluster_representatives(corpus)                 # coarse index: one node per cluster
    rep_rows = x[reps.long()].contiguous()
    out = {b: (torch.empty(b, K, dtype=torch.int32, device=dev), torch.empty(b, K, device=dev))
           for b in (B_SMALL, B_LARGE)}
    g_ids, g_sc = torch.empty(B_LARGE, K, dtype=torch.int32, device=dev), torch.empty(B_LARGE, K, device=dev)
    c_ids, c_sc = torch.empty(B_LARGE, 1, dtype=torch.int32, device=dev), torch.empty(B_LARGE, 1, device=dev)
    entries = torch.empty(B_LARGE, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] inputs ready after {time.time() - t_start:.0f} s")

    def leg_flat_small():
        ann.ann_flat_search_typed(x, q_small, K, ids=out[B_SMALL][0], scores=out[B_SMALL][1])

    def leg_flat_large():
        ann.ann_flat_search_typed(x, q_all, K, ids=out[B_LARGE][0], scores=out[B_LARGE][1])

    def nav_search(qq, ef, ids=None, scores=None):
        """Coarse entry search over the representatives, then the graph search from there."""
        B = qq.shape[0]
        ann.ann_flat_search_typed(rep_rows, qq, 1, ids=c_ids[:B], scores=c_sc[:B])
        ann.ann_gather_ids(reps, c_ids[:B].view(-1), out=entries[:B])
        return ann.ann_graph_search_entries_typed(x, graph_nav, entries[:B], qq, K, ef, ids=ids, scores=scores)

    leg_flat_large()
    torch.cuda.synchronize()
    exact = out[B_LARGE][0].cpu().numpy()                        # exact answers (checked against the oracle below)

    # ---- operating point: the cheapest ef with recall@3 >= 0.95 on the configuration's queries ----
    nav_table = []
    ef_op = args.ef
    for ef in (EF_CANDIDATES if args.ef == 0 else (args.ef,)):
        ids, _ = nav_search(q_all, ef)
        torch.cuda.synchronize()
        ms = timed(lambda: nav_search(q_all, ef), n=2 if ef >= 4096 else 4, w=0)
        nav_table.append({"ef": ef, "B": B_LARGE, "ms": ms, "qps": B_LARGE / ms * 1e3, "recall_at_3": recall3(ids, exact)})
        log(f"[bench] navigable graph ef={ef}: {ms:.2f} ms, recall@3 {nav_table[-1]['recall_at_3']:.4f}")
        if args.ef == 0 and nav_table[-1]["recall_at_3"] >= RECALL_TARGET:
            ef_op = ef
            break
    target_met = any(r["recall_at_3"] >= RECALL_TARGET for r in nav_table)
    if ef_op == 0:                                               # never reached: report the best recall seen
        ef_op = max(nav_table, key=lambda r: r["recall_at_3"])["ef"]

    def leg_graph():
        nav_search(q_all, ef_op, ids=g_ids, scores=g_sc)

    legs = (("flat_b16", leg_flat_small), ("flat_b512", leg_flat_large), ("graph_b512", leg_graph))

    def step(events=None):
        for i, (_, fn) in enumerate(legs):
            if events is not None:
                events[i][0].record()
            fn()
            if events is not None:
                events[i][1].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the library brackets its main kernels with HIP events on the launch stream while this is on
    ann.ann_timing_enable(True)

    # ---- timed region: exactly `steps` steps, bracketed by synchronize ---------------------
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in legs]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ann.ann_timing_enable(False)
    ms_per_step = wall * 1e3 / args.steps
    # average duration of one launch of each leg's main kernel (events on the launch stream).  The
    # graph leg's coarse entry search is a second matrix-core launch per step: taken out by position.
    stream_ms = ann.ann_timing_read_each(ann.binding.KERNEL_FLAT_STREAM)
    wide_ms = ann.ann_timing_read_each(ann.binding.KERNEL_FLAT_WIDE)
    graph_ms = ann.ann_timing_read_each(ann.binding.KERNEL_GRAPH)
    assert len(stream_ms) == args.steps and len(wide_ms) == 2 * args.steps and len(graph_ms) == args.steps, \
        (len(stream_ms), len(wide_ms), len(graph_ms))
    kernel_ms = {"flat_b16": sum(stream_ms) / args.steps, "flat_b512": sum(wide_ms[0::2]) / args.steps,
                 "graph_b512": sum(graph_ms) / args.steps}
    coarse_ms = sum(wide_ms[1::2]) / args.steps
    kernel_of_leg = {"flat_b16": "flat_stream_kernel", "flat_b512": "flat_wide_kernel", "graph_b512": "graph_search_kernel"}
    leg_ms = [sum(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)) / args.steps
              for i in range(len(legs))]
    value = B_LARGE / (leg_ms[2] * 1e-3)                         # graph queries/s at the operating point
    gpu_g = g_ids.cpu().numpy()
    recall_op = recall3(gpu_g, exact)
    log(f"[bench] timed region done after {time.time() - t_start:.0f} s: graph leg {leg_ms[2]:.2f} ms at ef={ef_op}, "
        f"recall@3 {recall_op:.4f}")

    # ---- oracle side: counters for the graph roofline, parity checks, CPU baseline -------------
    flat_bytes = float(N) * d * 2
    flat_flops = 2.0 * B_LARGE * N * d
    graph_bytes = None
    cpu_baseline = None
    checks = {}
    if not args.no_cpu:
        import oracle
        xh, qh, gh = x.cpu().numpy(), q_all.cpu().numpy(), graph_nav.cpu().numpy()
        eh = entries.cpu().numpy()
        n_flat = 128                                 # bounded sample of the flat legs (about 4 s of CPU work)
        t = time.perf_counter()
        o_f = oracle.flat_search(xh, qh[:n_flat], K)
        t_flat = (time.perf_counter() - t) / n_flat
        checks["flat_ids_equal_oracle_on_sample"] = float((exact[:n_flat] == o_f[0]).all(axis=1).mean())
        # graph leg: the oracle from the same entries on all queries (also gives the algorithmic bytes)
        t = time.perf_counter()
        o_g = oracle.graph_search(xh, gh, 0, qh, K, ef_op, entries=eh)
        t_graph = (time.perf_counter() - t) / B_LARGE
        n_dist, n_expand = o_g[3], o_g[4]
        graph_bytes = float((n_dist * d * 2 + n_expand * R * 4).sum())
        checks["graph_ids_equal_oracle"] = float((gpu_g == o_g[0]).all(axis=1).mean())
        checks["graph_oracle_nodes_scored_per_query"] = float(n_dist.mean())
        checks["graph_oracle_expansions_per_query"] = float(n_expand.mean())
        o_c = oracle.flat_search(xh[reps.cpu().numpy()], qh, 1)
        checks["coarse_entries_equal_oracle"] = float((reps.cpu().numpy()[o_c[0][:, 0]] == eh).mean())
        cpu_step = t_flat * (B_SMALL + B_LARGE) + t_graph * B_LARGE
        cpu_baseline = {
            "value": 1.0 / t_graph, "unit": "queries/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"graph oracle at the same operating point (ef={ef_op}, same entries) on all {B_LARGE} queries: "
                      f"{t_graph * 1e3:.1f} ms/query on all cores; flat oracle on {n_flat} queries: {t_flat * 1e3:.0f} ms/query",
            "flat_queries_per_s": 1.0 / t_flat,
            "whole_step_queries_per_s": (B_SMALL + 2 * B_LARGE) / cpu_step,
        }
        log(f"[bench] oracle legs done after {time.time() - t_start:.0f} s")

    rooflines = {
        "flat_b16": {"bound": "hbm", "achieved": flat_bytes / kernel_ms["flat_b16"] / 1e6, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "workload": "cfg1 N=1,000,000 d=768 fp16, B=16, k=3"},
        "flat_b512": {"bound": "mfma", "achieved": flat_flops / kernel_ms["flat_b512"] / 1e9,
                      "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "workload": "cfg1 N=1,000,000 d=768 fp16, B=512, k=3"},
        "graph_b512": {"bound": "hbm", "achieved": (graph_bytes / kernel_ms["graph_b512"] / 1e6) if graph_bytes else None,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "workload": f"cfg2 corpus and queries, navigable graph, per-query entries, B=512, ef={ef_op}, k=3",
                       "algorithmic_bytes": graph_bytes, "coarse_entry_search_ms": coarse_ms},
    }
    rooflines["flat_b512"]["target"] = "0.50 of peak"
    rooflines["flat_b16"]["target"] = "0.70 of peak"
    traffic = measured_traffic()
    for i, (leg, r) in enumerate(rooflines.items()):
        r["frac"] = r["achieved"] / r["peak"] if r["achieved"] is not None else None
        r["kernel"] = kernel_of_leg[leg]
        r["kernel_ms"] = kernel_ms[leg]
        r["leg_ms"] = leg_ms[i]
        r["leg_frac"] = r["frac"] * kernel_ms[leg] / leg_ms[i] if r["frac"] is not None else None
        # (the committed graph figure is for ef = 8192, the operating point the sweep finds on this workload)
        r["traffic"] = traffic.get(kernel_of_leg[leg]) if (leg != "graph_b512" or ef_op == 8192) else None
        r["traffic_source"] = (f"{TRAFFIC_FILE}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this command, "
                               "committed; not measured in this run") if r["traffic"] is not None else None
    rooflines["flat_b512"]["target_met"] = bool(rooflines["flat_b512"]["frac"] >= 0.50)
    rooflines["flat_b16"]["target_met"] = bool(rooflines["flat_b16"]["frac"] >= 0.70)
    dominant = max(range(len(legs)), key=lambda i: kernel_ms[legs[i][0]])
    roofline = dict(rooflines[legs[dominant][0]])
    roofline["leg"] = legs[dominant][0]

    # context numbers (not targets, not part of any fraction above): what the matrix cores of this machine
    # sustain on register operands, and the vendor GEMM for the same contraction without any top-k
    context = {"box_mfma_rate_TFLOPs": {"constant_operands": ann.ann_measure_mfma_rate(False),
                                        "random_operands": ann.ann_measure_mfma_rate(True)}}
    s_out = torch.empty(N, B_LARGE, dtype=x.dtype, device=dev)
    qt = q_all.t()
    gemm_ms = timed(lambda: torch.matmul(x, qt, out=s_out), n=10, w=3)
    del s_out
    context["vendor_gemm_same_shape"] = {"ms": gemm_ms, "TFLOPs": flat_flops / gemm_ms / 1e9,
                                         "note": "torch.matmul, writes S[N,B], no top-k; comparison only"}
    context["paper"] = "0.16 s ANN retrieval per sequence at efSearch 10 000 over 21 M x 384 on 22 CPU cores (Section 4.3); other hardware, other data"

    # ---- further legs, same run, outside the timed step: configurations 3 and 4 ---------------
    large = None
    if not args.no_large:
        large = {}
        c3 = synth.workload_corpus(3, device=dev)
        n3 = c3.x.shape[0]
        q3 = synth.make_queries(c3, 256)
        bytes3 = float(n3) * d * 2
        for B in (1, 16, 256):
            qb = q3[:B].contiguous()
            ann.ann_timing_enable(True)
            ms = timed(lambda: ann.ann_flat_search_typed(c3.x, qb, K), n=6, w=1)
            ann.ann_timing_enable(False)
            code = ann.binding.KERNEL_FLAT_WIDE if B >= 65 else ann.binding.KERNEL_FLAT_STREAM
            per = ann.ann_timing_read_each(code)
            k_ms = sum(per[1:]) / max(1, len(per) - 1)
            flops = 2.0 * B * n3 * d
            large[f"cfg3_flat_b{B}"] = {
                "workload": f"cfg3 N=21,000,000 d=768 fp16 (32.3 GB), B={B}, k=3", "call_ms": ms, "kernel_ms": k_ms,
                "qps": B / ms * 1e3, "hbm_GBs": bytes3 / k_ms / 1e6, "hbm_frac": bytes3 / k_ms / 1e6 / HBM_PEAK_GBS,
                "mfma_TFLOPs": flops / k_ms / 1e9, "mfma_frac": flops / k_ms / 1e9 / MFMA_F16_PEAK_TFLOPS,
                "bound": "hbm", "frac": bytes3 / k_ms / 1e6 / HBM_PEAK_GBS}
        if not args.no_cpu:
            n_s = 8                                  # the oracle needs about 0.7 s per query here
            ids3, _ = ann.ann_flat_search_typed(c3.x, q3, K)
            x3h = c3.x.cpu().numpy()
            t = time.perf_counter()
            o3 = oracle.flat_search(x3h, q3[:n_s].cpu().numpy(), K)
            large["cfg3_oracle"] = {"queries": n_s, "ms_per_query": (time.perf_counter() - t) / n_s * 1e3, "cores": oracle.threads(),
                                    "ids_equal_gpu": float((ids3[:n_s].cpu().numpy() == o3[0]).all(axis=1).mean())}
            del x3h
        del c3, q3
        torch.cuda.empty_cache()
        log(f"[bench] configuration 3 legs done after {time.time() - t_start:.0f} s")
        c4 = synth.workload_corpus(4, device=dev)
        q4 = synth.make_queries(c4, 256)
        g4 = synth.knn_graph_cluster_restricted(c4, 32, 8)
        e4 = synth.mean_entry(c4.x)
        ex4 = ann.ann_flat_search_typed(c4.x, q4, K)[0].cpu().numpy()
        if not args.no_cpu:
            x4h, g4h, q4h = c4.x.cpu().numpy(), g4.cpu().numpy(), q4.cpu().numpy()
        for ef in (32, 64, 128):
            ann.ann_timing_enable(True)
            ms = timed(lambda: ann.ann_graph_search_typed(c4.x, g4, e4, q4, K, ef), n=6, w=1)
            ann.ann_timing_enable(False)
            per = ann.ann_timing_read_each(ann.binding.KERNEL_GRAPH)
            k_ms = sum(per[1:]) / max(1, len(per) - 1)
            ids4 = ann.ann_graph_search_typed(c4.x, g4, e4, q4, K, ef)[0]
            row = {"workload": f"cfg4 N=10,000,000 d=768 fp16, literal graph R=32 and entry, B=256, ef={ef}, k=3",
                   "call_ms": ms, "kernel_ms": k_ms, "qps": 256 / ms * 1e3, "recall_at_3": recall3(ids4, ex4),
                   "recall_target_met": False, "bound": "hbm"}
            if not args.no_cpu:
                t = time.perf_counter()
                o4 = oracle.graph_search(x4h, g4h, e4, q4h, K, ef)
                row["oracle_ms_per_query"] = (time.perf_counter() - t) / 256 * 1e3
                b4 = float((o4[3] * d * 2 + o4[4] * 32 * 4).sum())
                row.update({"algorithmic_bytes": b4, "hbm_GBs": b4 / k_ms / 1e6, "frac": b4 / k_ms / 1e6 / HBM_PEAK_GBS,
                            "ids_equal_oracle": float((ids4.cpu().numpy() == o4[0]).all(axis=1).mean())})
            row["recall_target_met"] = bool(row["recall_at_3"] >= RECALL_TARGET)
            large[f"cfg4_graph_ef{ef}"] = row
        del c4, q4, g4
        torch.cuda.empty_cache()
        log(f"[bench] configuration 4 legs done after {time.time() - t_start:.0f} s")

    # ---- untimed report: per-B flat rates, per-ef graph rates and recall ---------------------
    sweep = None
    if not args.no_sweep:
        sweep = {"flat": [], "graph_literal": [], "graph_navigable": nav_table}
        for B in (1, 16, 64, 256, 512):
            qb = q_all[:B].contiguous()
            ms = timed(lambda: ann.ann_flat_search_typed(x, qb, K))
            sweep["flat"].append({"B": B, "ms": ms, "qps": B / ms * 1e3, "hbm_GBs": flat_bytes / ms / 1e6,
                                  "hbm_frac": flat_bytes / ms / 1e6 / HBM_PEAK_GBS,
                                  "mfma_TFLOPs": 2.0 * B * N * d / ms / 1e9,
                                  "mfma_frac": 2.0 * B * N * d / ms / 1e9 / MFMA_F16_PEAK_TFLOPS})
        # the paper retrieves k = 5 (Appendix B.3); batches between the configuration's sizes too
        sweep["flat_other"] = []
        for B, kk in ((1, 5), (16, 5), (128, 3), (128, 5), (512, 5), (512, 16)):
            qb = q_all[:B].contiguous()
            ms = timed(lambda: ann.ann_flat_search_typed(x, qb, kk))
            sweep["flat_other"].append({"B": B, "k": kk, "ms": ms, "qps": B / ms * 1e3, "hbm_GBs": flat_bytes / ms / 1e6,
                                        "mfma_TFLOPs": 2.0 * B * N * d / ms / 1e9})
        # configuration 2 as written: literal graph, one shared entry.  No ef reaches the recall target
        # (no edges between clusters); rates and recall for every listed (ef, B)
        for ef in (8, 16, 32, 64, 128, 256, 1024, 16384):
            for B in (1, 64, 512) if ef <= 256 else (512,):
                qb = q_all[:B].contiguous()
                ms = timed(lambda: ann.ann_graph_search_typed(x, graph, entry, qb, K, ef), n=5 if ef <= 1024 else 1, w=1)
                ids, _ = ann.ann_graph_search_typed(x, graph, entry, qb, K, ef)
                sweep["graph_literal"].append({"ef": ef, "B": B, "ms": ms, "qps": B / ms * 1e3,
                                               "recall_at_3": recall3(ids, exact), "recall_target_met": False})
        # larger batches than one resident round of workgroups, at the configuration's ef = 64
        sweep["graph_batch"] = []
        for Bx in (256, 512, 1024, 2048, 4096):
            qx = q_all.repeat((Bx + B_LARGE - 1) // B_LARGE, 1)[:Bx].contiguous()
            ms = timed(lambda: ann.ann_graph_search_typed(x, graph, entry, qx, K, 64), n=5, w=1)
            sweep["graph_batch"].append({"ef": 64, "B": Bx, "ms": ms, "qps": Bx / ms * 1e3})
        # the operating point with more queries than one resident round (2 workgroups per compute unit):
        # a workgroup slot takes the next query when its own ends, so the batch no longer waits for its
        # slowest query with every other slot idle (queries: copies of the configuration's 512)
        sweep["graph_navigable_batch"] = []
        for Bx in (1024, 2048):
            qx = q_all.repeat(Bx // B_LARGE, 1).contiguous()
            def nav_search_batch():
                cid_x, _ = ann.ann_flat_search_typed(rep_rows, qx, 1)
                return ann.ann_graph_search_entries_typed(x, graph_nav, ann.ann_gather_ids(reps, cid_x.view(-1)), qx, K, ef_op)
            ms = timed(nav_search_batch, n=1, w=1)
            sweep["graph_navigable_batch"].append({"ef": ef_op, "B": Bx, "ms": ms, "qps": Bx / ms * 1e3})
        # the rest of the navigable-graph table beyond the operating point, and a variant with little
        # query noise (std 0.05 / sqrt(d): NOT the configuration's queries)
        have = {r["ef"] for r in nav_table}
        for ef in (64, 256) + tuple(e for e in EF_CANDIDATES if e not in have):
            ms = timed(lambda: nav_search(q_all, ef), n=2 if ef >= 4096 else 4, w=1)
            ids, _ = nav_search(q_all, ef)
            nav_table.append({"ef": ef, "B": B_LARGE, "ms": ms, "qps": B_LARGE / ms * 1e3, "recall_at_3": recall3(ids, exact)})
        nav_table.sort(key=lambda r: r["ef"])
        qv = synth.make_queries(corpus, B_LARGE, noise_std=0.05 / math.sqrt(d))
        ex_v = ann.ann_flat_search_typed(x, qv, K)[0].cpu().numpy()
        sweep["graph_navigable_small_noise_variant"] = []
        for ef in (64, 256, 512, 1024):
            ms = timed(lambda: nav_search(qv, ef), n=3, w=1)
            sweep["graph_navigable_small_noise_variant"].append(
                {"queries": "noise std 0.05/sqrt(d) (labelled variant)", "ef": ef, "B": B_LARGE, "ms": ms,
                 "qps": B_LARGE / ms * 1e3, "recall_at_3": recall3(nav_search(qv, ef)[0], ex_v)})

        # Maturity (non-stall) exit, tau = 0.9, window 500, engine always ready, on the operating point's inputs
        sweep["nonstall"] = []
        cid, _ = ann.ann_flat_search_typed(rep_rows, q_all, 1)
        ent = ann.ann_gather_ids(reps, cid.view(-1))
        for ef in sorted({256, 1024, ef_op}):
            def run_ns():
                return ann.ann_graph_search_nonstall_typed(x, graph_nav, 0, q_all, K, ef, entries=ent, tau=0.9, window=500)

            def run_nat():
                return ann.ann_graph_search_nonstall_typed(x, graph_nav, 0, q_all, K, ef, entries=ent, tau=float("inf"))
            ms, ms_nat = timed(run_ns, n=2, w=1), timed(run_nat, n=2, w=1)
            a, b_ = run_ns(), run_nat()
            sweep["nonstall"].append({
                "setup": "navigable graph, coarse entries, the configuration's queries", "ef": ef, "B": B_LARGE,
                "ms": ms, "ms_natural_stop": ms_nat,
                "early_exit_fraction": float(a[2][:, 0].float().mean()),
                "expansions": float(a[2][:, 2].float().mean()),
                "expansions_natural_stop": float(b_[2][:, 2].float().mean()),
                "recall_at_3": recall3(a[0], exact), "recall_at_3_natural_stop": recall3(b_[0], exact)})
        # the two readings of "best and worst currently in the list" (Section 3.3), oracle against oracle
        if not args.no_cpu:
            sweep["rq_forms"] = []
            n_q = 128
            for ef in (256, 1024):
                forms = {}
                for form in ("node", "expansion"):
                    o = oracle.graph_search_nonstall(xh, gh, 0, qh[:n_q], K, ef, tau=0.9, window=500, form=form, entries=eh[:n_q])
                    forms[form] = o
                sa, sb = forms["node"][3], forms["expansion"][3]
                sweep["rq_forms"].append({
                    "ef": ef, "queries": n_q, "tau": 0.9, "window": 500,
                    "early_exit_fraction": {"node": float(sa[:, 0].mean()), "expansion": float(sb[:, 0].mean())},
                    "mean_expansions": {"node": float(sa[:, 2].mean()), "expansion": float(sb[:, 2].mean())},
                    "queries_leaving_at_another_expansion": int((sa[:, 2] != sb[:, 2]).sum()),
                    "mean_abs_difference_in_expansions": float(np.abs(sa[:, 2] - sb[:, 2]).mean()),
                    "recall_at_3": {"node": recall3(forms["node"][0], exact[:n_q]), "expansion": recall3(forms["expansion"][0], exact[:n_q])}})

    result = {
        "metric": METRIC, "value": value, "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "value_definition": f"graph leg of the step: {B_LARGE} queries / {leg_ms[2]:.3f} ms (coarse entry search + graph search, "
                            f"ef={ef_op}), the cheapest swept search range with recall@3 >= {RECALL_TARGET}",
        "graph_recall_at_3": recall_op, "graph_recall_target_met": bool(recall_op >= RECALL_TARGET and target_met),
        "graph_operating_point": {"ef": ef_op, "graph": "cfg2 graph with half of each row replaced by reverse edges (R=32)",
                                  "entry": "per query: best of one representative per cluster (exact search, part of the leg)",
                                  "queries": "the configuration's own (noise std 0.05 per coordinate)"},
        "literal_cfg2_recall_target_met": False,
        "config": {"workload": "cfg1 flat + cfg2 graph: N=1,000,000 d=768 fp16 storage / fp32 accumulate, 1024-cluster Zipf(1.1) "
                               f"mixture, seed 1; step = flat B=16 + flat B=512 + graph B=512 at ef={ef_op}; further legs outside "
                               "the step: cfg3 flat N=21,000,000 B=1/16/256, cfg4 graph N=10,000,000 B=256 ef=32/64/128",
                   "N": N, "d": d, "k": K, "R": R, "ef": ef_op, "queries_per_step": B_SMALL + 2 * B_LARGE},
        "legs": {legs[i][0]: {"ms": leg_ms[i], "qps": (B_SMALL if i == 0 else B_LARGE) / leg_ms[i] * 1e3} for i in range(len(legs))},
        "flat_targets": {"hbm_frac_b16": rooflines["flat_b16"]["frac"], "hbm_target_0.70_met": rooflines["flat_b16"]["target_met"],
                         "mfma_frac_b512": rooflines["flat_b512"]["frac"], "mfma_target_0.50_met": rooflines["flat_b512"]["target_met"]},
        "checks": checks,
        "roofline": roofline, "rooflines": rooflines, "large_configs": large, "cpu_baseline": cpu_baseline,
        "context": context, "sweep": sweep,
    }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
