"""The paper-shaped retrieval workload on one GPU: 21 M passages x 384 dimensions (the size of
the chunked-Wikipedia index embedded by a 384-d encoder, Appendix B.3), a graph index with at
most 32 neighbours per node, search ranges (candidate-list sizes) up to 10 000 (Section 4.3 /
Appendix B.3), top-k with k = 5.

    python -m paper_2505_12065_amd.paper_shape [--scale 0.1] [--queries 512]

Synthetic stand-in data (clustered Gaussian mixture, see synth.py), so recall numbers describe
this generator, not the paper's corpus.  Prints one JSON line per search range: queries/s of
the whole call (coarse entry search + graph search) and recall@5 against the library's own
exact search.  Everything runs in the library's kernels; torch only generates the inputs.
"""
from __future__ import annotations

import argparse
import json
import math
import sys
import time

import torch

from . import synth
from .binding import (ann_flat_search_typed, ann_gather_ids, ann_graph_search_entries_typed,
                      ann_graph_search_nonstall_typed)

K = 5
N_FULL, D, C_FULL, SEED = 21_000_000, 384, 4096, 5


def recall(ids: torch.Tensor, ref: torch.Tensor) -> float:
    a, b = ids.cpu().numpy(), ref.cpu().numpy()
    return sum(len(set(a[i].tolist()) & set(b[i].tolist())) for i in range(a.shape[0])) / a.size


def timed(fn, n=3):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--scale", type=float, default=1.0, help="fraction of the 21 M rows (and of the 4096 clusters)")
    ap.add_argument("--queries", type=int, default=512)
    ap.add_argument("--ef", type=int, nargs="*", default=[64, 256, 1024, 4096, 10000])
    ap.add_argument("--query-noise", type=float, default=0.05 / math.sqrt(D),
                    help="per-coordinate std of the query noise (0.05 is the literal value of the workload table)")
    args = ap.parse_args()
    dev = "cuda:0"
    N = max(4096, int(round(N_FULL * args.scale)))
    C = max(8, int(round(C_FULL * args.scale)))
    t = time.time()
    corpus = synth.make_corpus(N, D, C, SEED, sigma=(0.2, 0.5), zipf_a=1.1, dtype=torch.float16, device=dev)
    x = corpus.x
    q = synth.make_queries(corpus, args.queries, noise_std=args.query_noise)
    torch.cuda.synchronize()
    print(f"corpus {N} x {D} fp16 ({x.numel() * 2 / 1e9:.2f} GB), {C} clusters: {time.time() - t:.1f} s", file=sys.stderr, flush=True)
    t = time.time()
    graph = synth.with_reverse_edges(synth.knn_graph_cluster_restricted(corpus, 32, 8, progress=True), x)
    reps = synth.cluster_representatives(corpus)
    rep_rows = x[reps.long()].contiguous()
    torch.cuda.synchronize()
    print(f"graph (32 slots: 16-NN + reverse edges) and {reps.numel()} representatives: {time.time() - t:.1f} s",
          file=sys.stderr, flush=True)

    exact, _ = ann_flat_search_typed(x, q, K)
    flat_ms = timed(lambda: ann_flat_search_typed(x, q, K))
    print(json.dumps({"search": "flat (exact)", "N": N, "d": D, "B": args.queries, "k": K, "ms": flat_ms,
                      "qps": args.queries / flat_ms * 1e3}), flush=True)
    for ef in args.ef:
        def run():
            cid, _ = ann_flat_search_typed(rep_rows, q, 1)
            ent = ann_gather_ids(reps, cid.view(-1))
            return ann_graph_search_entries_typed(x, graph, ent, q, K, ef)
        ms = timed(run, n=2 if ef >= 4096 else 3)
        ids, _ = run()
        line = {"search": "graph", "N": N, "d": D, "R": 32, "ef": ef, "B": args.queries, "k": K, "ms": ms,
                "qps": args.queries / ms * 1e3, "ms_per_query_alone": None, f"recall_at_{K}": recall(ids, exact)}
        # one query on its own: the latency a single retrieval call of the agent sees
        q1 = q[:1].contiguous()

        def run1():
            cid, _ = ann_flat_search_typed(rep_rows, q1, 1)
            return ann_graph_search_entries_typed(x, graph, ann_gather_ids(reps, cid.view(-1)), q1, K, ef)
        line["ms_per_query_alone"] = timed(run1, n=2)
        # maturity exit at the paper's settings
        cid, _ = ann_flat_search_typed(rep_rows, q, 1)
        ent = ann_gather_ids(reps, cid.view(-1))
        ns = ann_graph_search_nonstall_typed(x, graph, 0, q, K, ef, entries=ent, tau=0.9, window=500)
        line["nonstall_tau0.9"] = {"early_exit_fraction": float(ns[2][:, 0].float().mean()),
                                   "expansions": float(ns[2][:, 2].float().mean()),
                                   f"recall_at_{K}": recall(ns[0], exact)}
        print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
