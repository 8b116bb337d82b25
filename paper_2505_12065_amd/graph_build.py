"""Proximity-graph rows built with the library's own exact search (the graph index of Section 2.1 /
Appendix B.3 is built offline from the passage embeddings; here its k-NN rows come from the flat-scan
kernels of this library instead of a separate builder).

    python -m paper_2505_12065_amd.graph_build        # times the build of the 1 M x 768 workload graph

`knn_rows_by_cluster` computes, for every point, its R best neighbours by inner product inside the pool
"all points of the n_near clusters whose normalised centroid is most similar to the point" (the graph
of the workload table), self excluded, ties to the lower id, short pools padded with -1:

  * per cluster b: corpus = the rows of b's members, queries = the rows of every point whose pool holds b;
    R + 1 results are needed per query (the point itself may be among them) but one call returns at most
    ANN_K_MAX = 16, so the rows come in pages of 16 through `ann_flat_search_after_typed`, each page
    continuing after the last pair of the one before;
  * per point: the best R of the candidates of its n_near clusters, under the library's order.

Only the assignment of points to clusters (a small N x C product) and the final few-way merges run in
torch; every point-to-point score and every top-k selection runs in the library's kernels.
"""
from __future__ import annotations

import math
import sys
import time
from typing import Optional

import torch

from .binding import ANN_K_MAX, ann_flat_search_typed


def knn_rows_by_cluster(x: torch.Tensor, labels: torch.Tensor, centroids: torch.Tensor, R: int, n_near: int = 8, *,
                        query_block: int = 8192, progress: bool = False) -> torch.Tensor:
    """x [N, d] fp16/bf16/fp32 on the GPU, labels [N] (cluster of each point), centroids [C, d] fp32.
    Returns int32 [N, R] on x's device."""
    dev = x.device
    N = x.shape[0]
    C = centroids.shape[0]
    n_near = min(n_near, C)
    labels = labels.to(dev).long()
    cn = (centroids / centroids.norm(dim=1, keepdim=True)).to(dev)
    near = torch.empty(N, n_near, dtype=torch.int64, device=dev)
    for r0 in range(0, N, 1 << 17):
        near[r0:r0 + (1 << 17)] = torch.topk(x[r0:r0 + (1 << 17)].float() @ cn.T, n_near, dim=1).indices
    order = torch.argsort(labels, stable=True)                   # members of a cluster, ids ascending
    counts = torch.bincount(labels, minlength=C)
    starts = (torch.cumsum(counts, 0) - counts).tolist()
    counts = counts.tolist()
    # the points whose pool holds cluster b, ids ascending: the (point, cluster) pairs ordered by cluster
    pair_cluster = near.flatten()
    pair_order = torch.argsort(pair_cluster, stable=True)
    ask_counts = torch.bincount(pair_cluster, minlength=C)
    ask_starts = (torch.cumsum(ask_counts, 0) - ask_counts).tolist()
    ask_counts = ask_counts.tolist()
    pair_point = pair_order // n_near                            # (a point names a cluster at most once)
    pages = (R + 1 + ANN_K_MAX - 1) // ANN_K_MAX
    best_s = torch.full((N, R), -math.inf, dtype=torch.float32, device=dev)
    best_i = torch.full((N, R), -1, dtype=torch.int64, device=dev)
    last = time.time()
    for b in range(C):
        nb = counts[b]
        if nb == 0:
            continue
        members = order[starts[b]: starts[b] + nb]
        rows = x[members].contiguous()
        askers = pair_point[ask_starts[b]: ask_starts[b] + ask_counts[b]]
        if progress and time.time() - last > 20:
            print(f"  graph build: cluster {b}/{C} ({nb} members, {askers.numel()} queries)", file=sys.stderr, flush=True)
            last = time.time()
        k = min(ANN_K_MAX, nb)
        for a0 in range(0, askers.numel(), query_block):
            a = askers[a0:a0 + query_block]
            q = x[a].contiguous()
            got_s, got_i, after = [], [], None
            for _ in range(pages):
                idx, sc = ann_flat_search_typed(rows, q, k, after=after)
                got_s.append(sc)
                got_i.append(idx)
                if k < ANN_K_MAX:
                    break                                        # the whole cluster fitted in one page
                after = (sc[:, -1].contiguous(), idx[:, -1].contiguous())
            sc = torch.cat(got_s, 1)
            idx = torch.cat(got_i, 1).long()
            ids = torch.where(idx >= 0, members[idx.clamp(min=0)], torch.full_like(idx, -1))
            drop = (ids < 0) | (ids == a[:, None])               # padding, and the point itself
            sc = torch.where(drop, torch.full_like(sc, -math.inf), sc)
            ids = torch.where(drop, torch.full_like(ids, -1), ids)
            # merge with what the point has from its other clusters: score descending, id ascending
            all_s = torch.cat([best_s[a], sc], 1)
            all_i = torch.cat([best_i[a], ids], 1)
            key = torch.where(all_i < 0, torch.full_like(all_i, 1 << 62), all_i)
            o = torch.argsort(key, dim=1, stable=True)
            all_s, all_i = torch.gather(all_s, 1, o), torch.gather(all_i, 1, o)
            o = torch.argsort(all_s, dim=1, descending=True, stable=True)
            best_s[a] = torch.gather(all_s, 1, o)[:, :R]
            best_i[a] = torch.gather(all_i, 1, o)[:, :R]
    return best_i.to(torch.int32)


def main(argv: Optional[list] = None) -> int:
    from . import synth
    scale = float(argv[0]) if argv else 1.0
    corpus = synth.workload_corpus(2, device="cuda:0", scale=scale)
    torch.cuda.synchronize()
    t = time.time()
    g = knn_rows_by_cluster(corpus.x, corpus.labels, corpus.centroids, 32, 8, progress=True)
    torch.cuda.synchronize()
    t_lib = time.time() - t
    t = time.time()
    ref = synth.knn_graph_cluster_restricted(corpus, 32, 8)
    torch.cuda.synchronize()
    t_ref = time.time() - t
    same = float((g == ref).all(dim=1).float().mean())
    print(f"N={corpus.x.shape[0]}: rows by the library's search {t_lib:.1f} s, by the generator's matmul + top-k {t_ref:.1f} s, "
          f"identical rows {same:.5f}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
