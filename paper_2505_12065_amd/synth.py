"""Seeded synthetic inputs for the retrieval hot path: clustered unit-norm
passage-embedding corpora, noisy queries, entry nodes and fixed-degree kNN graphs.

These stand in for the paper's chunked-Wikipedia index (about 21 M chunk
embeddings, graph index with up to 32 neighbours per node; Appendix B.3,
"Detailed Experimental Setup") and for its QA query sets, none of which can be
shipped.  Everything here is *input generation*: the outputs of this module are
handed unchanged both to the HIP library and to the CPU oracle.  Nothing in this
file is called by the search path, and the search path's own arithmetic (scoring
a query against the corpus, top-k selection, beam search) does not live here.
The graph builder uses plain torch matmul/top-k because a proximity graph is an
input of ``ann_graph_search``, exactly as the pre-built index is an input of the
paper's retriever.

Recipe (all randomness from ``torch.Generator`` seeded from ``seed``):

* centroids  c_r ~ N(0, I_d), r = 0..C-1 (not normalised)
* per-cluster spread sigma_r: a constant, or U[lo, hi]
* cluster sizes: equal (tiny case) or a deterministic Zipf(a) apportionment
  n_r = floor(N * r^-a / H), remainder given to the largest cluster
* labels are shuffled by a seeded permutation so the row id carries no cluster
  information
* point  x = c_label + sigma_label * N(0, I_d), L2-normalised in fp32, then
  rounded to the storage dtype (no re-normalisation after rounding)
* query  = a random corpus row (as stored) + N(0, noise_std^2) per coordinate,
  L2-normalised in fp32, rounded to the storage dtype
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import torch

_CHUNK_ROWS = 1 << 17


def _gen(seed: int, stream: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(stream) * 7919 + 12345) % (2**63 - 1))
    return g


def zipf_sizes(N: int, C: int, a: float = 1.1) -> torch.Tensor:
    """Deterministic apportionment of N points to C clusters, n_r proportional to r^-a."""
    r = torch.arange(1, C + 1, dtype=torch.float64)
    w = r.pow(-a)
    n = torch.floor(N * w / w.sum()).to(torch.int64)
    n[0] += N - int(n.sum())
    return n


def equal_sizes(N: int, C: int) -> torch.Tensor:
    n = torch.full((C,), N // C, dtype=torch.int64)
    n[: N % C] += 1
    return n


@dataclasses.dataclass
class Corpus:
    x: torch.Tensor          # [N, d] storage dtype, on `device`
    labels: torch.Tensor     # [N] int32 (cpu)
    centroids: torch.Tensor  # [C, d] fp32 (cpu), un-normalised
    sigmas: torch.Tensor     # [C] fp32 (cpu)
    seed: int


def make_corpus(N: int, d: int, C: int, seed: int, *, sigma=(0.2, 0.5),
                zipf_a: Optional[float] = 1.1, dtype=torch.float16,
                device: str = "cpu") -> Corpus:
    """Gaussian-mixture corpus, L2-normalised, stored as `dtype` on `device`.

    Cluster structure (centroids, spreads, labels) is always drawn on the CPU so
    it does not depend on the device; only the bulk per-point noise is drawn on
    `device`, in fixed-size row chunks with one generator per chunk.
    """
    g0 = _gen(seed, 0)
    centroids = torch.randn(C, d, generator=g0)
    if isinstance(sigma, (tuple, list)):
        lo, hi = sigma
        sigmas = lo + (hi - lo) * torch.rand(C, generator=g0)
    else:
        sigmas = torch.full((C,), float(sigma))
    sizes = zipf_sizes(N, C, zipf_a) if zipf_a is not None else equal_sizes(N, C)
    labels = torch.repeat_interleave(torch.arange(C, dtype=torch.int32), sizes)
    labels = labels[torch.randperm(N, generator=g0)]

    x = torch.empty(N, d, dtype=dtype, device=device)
    cen_dev = centroids.to(device)
    sig_dev = sigmas.to(device)
    for ci, r0 in enumerate(range(0, N, _CHUNK_ROWS)):
        r1 = min(N, r0 + _CHUNK_ROWS)
        lab = labels[r0:r1].to(device=device, dtype=torch.int64)
        g = _gen(seed, 1000 + ci, device)
        p = torch.randn(r1 - r0, d, generator=g, device=device)
        p = cen_dev[lab] + sig_dev[lab, None] * p
        p = p / p.norm(dim=1, keepdim=True)
        x[r0:r1] = p.to(dtype)
    return Corpus(x=x, labels=labels, centroids=centroids, sigmas=sigmas, seed=seed)


def make_queries(corpus: Corpus, B: int, *, noise_std: float = 0.05,
                 stream: int = 1) -> torch.Tensor:
    """B queries: random stored corpus rows plus per-coordinate Gaussian noise,
    renormalised in fp32 and rounded to the corpus dtype. Same device as the corpus."""
    x = corpus.x
    N, d = x.shape
    g = _gen(corpus.seed, 500 + stream)
    rows = torch.randint(0, N, (B,), generator=g)
    noise = torch.randn(B, d, generator=g)
    q = x[rows.to(x.device)].float() + noise_std * noise.to(x.device)
    q = q / q.norm(dim=1, keepdim=True)
    return q.to(x.dtype)


def mean_entry(x: torch.Tensor) -> int:
    """Row with the largest inner product with the fp64 mean of the stored corpus
    (ties: lower id)."""
    N = x.shape[0]
    mu = torch.zeros(x.shape[1], dtype=torch.float64, device=x.device)
    for r0 in range(0, N, _CHUNK_ROWS):
        mu += x[r0:r0 + _CHUNK_ROWS].double().sum(0)
    mu /= N
    best, best_id = -math.inf, 0
    for r0 in range(0, N, _CHUNK_ROWS):
        s = x[r0:r0 + _CHUNK_ROWS].double() @ mu
        m = float(s.max())
        if m > best:  # strict: an equal value in a later chunk has a higher id
            best = m
            best_id = r0 + int((s == m).nonzero()[0, 0])
    return best_id


def _scores(a: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    """fp32 inner products a @ b.T.  16-bit inputs on a GPU go through the matrix cores
    with fp32 output when torch offers that (exact products, fp32 accumulation); otherwise
    the operands are widened to fp32 first."""
    if a.is_cuda and a.dtype in (torch.float16, torch.bfloat16):
        try:
            return torch.mm(a, b.T, out_dtype=torch.float32)
        except (RuntimeError, TypeError):
            pass
    return a.float() @ b.float().T


def _topr_rows(scores: torch.Tensor, ids: torch.Tensor, R: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Best R per row by (score desc, id asc). `ids[j]` is the row id of column j,
    ascending. Rows with fewer than R finite scores are padded with id -1."""
    n_col = scores.shape[1]
    take = min(n_col, R + 8)
    v, j = torch.topk(scores, take, dim=1)
    cand = ids[j]
    # exact order inside the candidate window: stable sort by id, then by score
    o = torch.argsort(cand, dim=1, stable=True)
    v, cand = torch.gather(v, 1, o), torch.gather(cand, 1, o)
    o = torch.argsort(v, dim=1, descending=True, stable=True)
    v, cand = torch.gather(v, 1, o), torch.gather(cand, 1, o)
    if take > R:
        if take < n_col:
            # a tie that runs to the window edge could hide a lower id outside it:
            # redo those rows with a full stable sort (columns are in id order)
            edge_tie = ((v[:, R - 1] == v[:, take - 1]) & torch.isfinite(v[:, R - 1])).nonzero().flatten()
            if edge_tie.numel():
                fv, fj = torch.sort(scores[edge_tie], dim=1, descending=True, stable=True)
                v[edge_tie], cand[edge_tie] = fv[:, :take], ids[fj[:, :take]]
        v, cand = v[:, :R], cand[:, :R]
    cand = torch.where(torch.isfinite(v), cand, torch.full_like(cand, -1))
    if cand.shape[1] < R:
        pad = torch.full((cand.shape[0], R - cand.shape[1]), -1, dtype=cand.dtype, device=cand.device)
        padv = torch.full((v.shape[0], R - v.shape[1]), -math.inf, dtype=v.dtype, device=v.device)
        cand, v = torch.cat([cand, pad], 1), torch.cat([v, padv], 1)
    return v, cand


def knn_graph(x: torch.Tensor, R: int, *, row_block: int = 2048) -> torch.Tensor:
    """Exact directed R-NN graph by inner product over the whole corpus, self
    excluded, ties to the lower id. Returns int32 [N, R] on x's device."""
    N = x.shape[0]
    xf = x.float()
    ids = torch.arange(N, device=x.device)
    out = torch.empty(N, R, dtype=torch.int32, device=x.device)
    for r0 in range(0, N, row_block):
        r1 = min(N, r0 + row_block)
        s = xf[r0:r1] @ xf.T
        s[torch.arange(r1 - r0, device=x.device), torch.arange(r0, r1, device=x.device)] = -math.inf
        _, nb = _topr_rows(s, ids, R)
        out[r0:r1] = nb.to(torch.int32)
    return out


def knn_graph_cluster_restricted(corpus: Corpus, R: int, n_near: int = 8, *,
                                 row_block: int = 4096, col_block: int = 1 << 16,
                                 progress: bool = False) -> torch.Tensor:
    """Directed R-NN graph where point i's candidate pool is every point whose
    generator label is one of the `n_near` clusters whose L2-normalised centroid
    has the largest inner product with x_i. Self excluded, ties to the lower
    id, short pools padded with -1. Returns int32 [N, R] on the corpus device.
    """
    x = corpus.x
    dev = x.device
    N, _ = x.shape
    C = corpus.centroids.shape[0]
    n_near = min(n_near, C)
    cn = (corpus.centroids / corpus.centroids.norm(dim=1, keepdim=True)).to(dev)
    labels = corpus.labels.to(dev).long()
    near = torch.empty(N, n_near, dtype=torch.int64, device=dev)
    for r0 in range(0, N, _CHUNK_ROWS):
        s = x[r0:r0 + _CHUNK_ROWS].float() @ cn.T
        near[r0:r0 + _CHUNK_ROWS] = torch.topk(s, n_near, dim=1).indices
    order = torch.argsort(labels, stable=True)          # members of a cluster, ids ascending
    counts = torch.bincount(labels, minlength=C)
    starts = torch.cumsum(counts, 0) - counts

    best_v = torch.full((N, R), -math.inf, dtype=torch.float32, device=dev)
    best_i = torch.full((N, R), -1, dtype=torch.int64, device=dev)
    import time
    last = time.time()
    for b in range(C):
        nb = int(counts[b])
        if nb == 0:
            continue
        if progress and time.time() - last > 20:
            print(f"  graph build: cluster {b}/{C} ({nb} members)", flush=True)
            last = time.time()
        members = order[int(starts[b]): int(starts[b]) + nb]
        askers = (near == b).any(dim=1).nonzero().flatten()   # points whose pool contains cluster b
        if askers.numel() == 0:
            continue
        for a0 in range(0, askers.numel(), row_block):
            a = askers[a0:a0 + row_block]
            xa = x[a]
            cur_v, cur_i = best_v[a], best_i[a]
            for m0 in range(0, nb, col_block):
                m = members[m0:m0 + col_block]
                s = _scores(xa, x[m])
                s[a[:, None] == m[None, :]] = -math.inf
                v, i = _topr_rows(s, m, R)
                # merge the running best with this block's best, same total order
                allv, alli = torch.cat([cur_v, v], 1), torch.cat([cur_i, i], 1)
                alli_key = torch.where(alli < 0, torch.full_like(alli, 2**62), alli)
                o = torch.argsort(alli_key, dim=1, stable=True)
                allv, alli = torch.gather(allv, 1, o), torch.gather(alli, 1, o)
                o = torch.argsort(allv, dim=1, descending=True, stable=True)
                cur_v, cur_i = torch.gather(allv, 1, o)[:, :R], torch.gather(alli, 1, o)[:, :R]
            best_v[a], best_i[a] = cur_v, cur_i
    return best_i.to(torch.int32)


def cluster_representatives(corpus: Corpus) -> torch.Tensor:
    """One node per non-empty cluster: the member with the largest inner product with the
    cluster's L2-normalised centroid (ties: lower id).  int32, cluster order, corpus device.
    A coarse index for per-query entry nodes: search the representatives' rows exactly and
    start the graph search of a query at the best one."""
    x = corpus.x
    dev = x.device
    labels = corpus.labels.to(dev).long()
    cn = (corpus.centroids / corpus.centroids.norm(dim=1, keepdim=True)).to(dev)
    C = cn.shape[0]
    s = torch.empty(x.shape[0], dtype=torch.float32, device=dev)
    for r0 in range(0, x.shape[0], _CHUNK_ROWS):
        s[r0:r0 + _CHUNK_ROWS] = (x[r0:r0 + _CHUNK_ROWS].float() * cn[labels[r0:r0 + _CHUNK_ROWS]]).sum(1)
    best = torch.full((C,), -math.inf, device=dev).scatter_reduce(0, labels, s, reduce="amax")
    winners = (s == best[labels]).nonzero().flatten()            # ascending ids
    rep = torch.full((C,), -1, dtype=torch.int64, device=dev)
    rep.scatter_reduce_(0, labels[winners], winners, reduce="amin", include_self=False)
    return rep[rep >= 0].to(torch.int32)


def with_reverse_edges(graph: torch.Tensor, x: torch.Tensor, n_forward: Optional[int] = None, *,
                       row_block: int = 8192) -> torch.Tensor:
    """Same shape [N, R]: row j keeps its first `n_forward` (default R/2) neighbours, then takes the
    best nodes that name j in their own row (reverse neighbours, by score desc, id asc, those already
    kept skipped), then its remaining forward neighbours until R slots are full.  A standard way to
    make a directed k-NN graph easier to navigate at the same degree."""
    N, R = graph.shape
    dev = graph.device
    nf = R // 2 if n_forward is None else n_forward
    g = graph.long()
    # score of every edge i -> g[i, r]
    sc = torch.full((N, R), -math.inf, dtype=torch.float32, device=dev)
    for r0 in range(0, N, row_block):
        gi = g[r0:r0 + row_block]
        ok = gi >= 0
        nb = x[gi.clamp(min=0)].float()                           # [rows, R, d]
        sc[r0:r0 + row_block] = torch.where(ok, (nb * x[r0:r0 + row_block].float()[:, None, :]).sum(-1),
                                            torch.full_like(sc[r0:r0 + row_block], -math.inf))
    src = torch.arange(N, device=dev)[:, None].expand(N, R).reshape(-1)
    dst, val = g.reshape(-1), sc.reshape(-1)
    keep = dst >= 0
    src, dst, val = src[keep], dst[keep], val[keep]                # src ascending
    o = torch.argsort(val, descending=True, stable=True)
    src, dst = src[o], dst[o]
    o = torch.argsort(dst, stable=True)
    src, dst = src[o], dst[o]                                      # by dst, then score desc, then src asc
    counts = torch.bincount(dst, minlength=N)
    starts = torch.cumsum(counts, 0) - counts
    rank = torch.arange(dst.numel(), device=dev) - starts[dst]
    top = rank < R
    rev = torch.full((N, R), -1, dtype=torch.int64, device=dev)
    rev[dst[top], rank[top]] = src[top]
    out = torch.empty_like(graph)
    for r0 in range(0, N, row_block):
        cand = torch.cat([g[r0:r0 + row_block, :nf], rev[r0:r0 + row_block], g[r0:r0 + row_block, nf:]], 1)
        W = cand.shape[1]
        same = cand[:, :, None] == cand[:, None, :]                # [rows, W, W]
        earlier = torch.tril(torch.ones(W, W, dtype=torch.bool, device=dev), diagonal=-1)
        drop = (same & earlier).any(2) | (cand < 0)
        o = torch.argsort(drop.to(torch.int8), dim=1, stable=True)  # kept entries first, order preserved
        cand, drop = torch.gather(cand, 1, o), torch.gather(drop, 1, o)
        cand = torch.where(drop, torch.full_like(cand, -1), cand)
        out[r0:r0 + row_block] = cand[:, :R].to(graph.dtype)
    return out


def diversity_pruned(graph: torch.Tensor, x: torch.Tensor, keep: int, *, row_block: int = 4096) -> Tuple[torch.Tensor, float]:
    """The neighbour-selection heuristic of HNSW-style index builders applied to the rows of a k-NN graph
    (the rows are sorted best first): a candidate c of node i is taken only if it is closer to i than to every
    neighbour taken before it, score(c, i) > score(c, s) for all selected s; at most `keep` are taken, candidates
    passed over fill what is left of the `keep` slots (in their order), the other slots are -1.  Returns the
    pruned graph [N, R] (same shape) and the fraction of candidates the rule passed over.  Input preparation
    only: the graph is an input of the search."""
    N, R = graph.shape
    dev = graph.device
    out = torch.full_like(graph, -1)
    passed_over = 0
    total = 0
    for r0 in range(0, N, row_block):
        gi = graph[r0:r0 + row_block].long()
        ok = gi >= 0
        nb = x[gi.clamp(min=0)].float()                              # [rows, R, d]
        to_node = (nb * x[r0:r0 + row_block].float()[:, None, :]).sum(-1)   # score(c, i)
        among = torch.bmm(nb, nb.transpose(1, 2))                    # score(c, c')
        rows = gi.shape[0]
        taken = torch.zeros(rows, R, dtype=torch.bool, device=dev)
        closest_taken = torch.full((rows, R), -math.inf, device=dev)  # max over taken s of score(c, s)
        n_taken = torch.zeros(rows, dtype=torch.long, device=dev)
        for c in range(R):
            take = ok[:, c] & (to_node[:, c] > closest_taken[:, c]) & (n_taken < keep)
            taken[:, c] = take
            n_taken += take.long()
            closest_taken = torch.where(take[:, None], torch.maximum(closest_taken, among[:, :, c]), closest_taken)
        skipped = ok & ~taken
        passed_over += int(skipped.sum())
        total += int(ok.sum())
        # selected first, then the passed-over candidates, each group in its order, `keep` slots in all
        order = torch.argsort((~taken).to(torch.int8) + 2 * (~ok).to(torch.int8), dim=1, stable=True)
        cand = torch.gather(gi, 1, order)
        valid = torch.gather(ok, 1, order)
        cand = torch.where(valid & (torch.arange(R, device=dev)[None, :] < keep), cand, torch.full_like(cand, -1))
        out[r0:r0 + row_block] = cand.to(graph.dtype)
    return out, passed_over / max(1, total)


def ring_union(graph: torch.Tensor) -> torch.Tensor:
    """Append the two ring edges i -> i±1 (mod N) to every row: a strongly
    connected test graph for the 'ef >= N equals exact search' special case."""
    N = graph.shape[0]
    i = torch.arange(N, dtype=torch.int32, device=graph.device)
    return torch.cat([graph, ((i + 1) % N)[:, None], ((i - 1) % N)[:, None]], 1).contiguous()


# --- the five workload configurations -----------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    N: int
    d: int
    C: int
    seed: int
    dtype: torch.dtype
    sigma: object
    zipf_a: Optional[float]
    k: int
    R: int = 0


WORKLOADS = {
    0: Workload("cfg0-tiny", 10_000, 128, 16, 0, torch.float32, 0.3, None, 10, 16),
    1: Workload("cfg1-flat-1M", 1_000_000, 768, 1024, 1, torch.float16, (0.2, 0.5), 1.1, 3),
    2: Workload("cfg2-graph-1M", 1_000_000, 768, 1024, 1, torch.float16, (0.2, 0.5), 1.1, 3, 32),
    3: Workload("cfg3-flat-21M", 21_000_000, 768, 4096, 2, torch.float16, (0.2, 0.5), 1.1, 3),
    4: Workload("cfg4-graph-10M", 10_000_000, 768, 4096, 3, torch.float16, (0.2, 0.5), 1.1, 3, 32),
}


def workload_corpus(cfg: int, device: str = "cpu", *, scale: float = 1.0) -> Corpus:
    """Corpus of configuration `cfg`; `scale` < 1 shrinks N and C together for
    parity cases the CPU oracle must finish quickly."""
    w = WORKLOADS[cfg]
    N = max(64, int(round(w.N * scale)))
    C = max(4, int(round(w.C * scale))) if scale != 1.0 else w.C
    return make_corpus(N, w.d, C, w.seed, sigma=w.sigma, zipf_a=w.zipf_a, dtype=w.dtype, device=device)
