"""Comparison of a GPU top-k result with the oracle's, under the stated rule:
ids identical except for order swaps (and swaps across the rank-k boundary) among
entries whose oracle scores differ by less than `tol`; scores within `tol`."""
import numpy as np

import oracle

TOL = 1e-4   # absolute, on unit-norm vectors (spec tolerance)


def to_np(t):
    """torch tensor -> numpy array holding the same bits (bf16 as uint16)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def np_dtype_name(t):
    import torch
    return {torch.float16: "f16", torch.bfloat16: "bf16", torch.float32: "f32"}[t.dtype]


def compare_topk(g_ids, g_sc, o_ids, o_sc64, corpus_np, queries_np, dtype=None, tol=TOL, rows=None):
    """Returns (n_strict, n_tolerant, n_queries); raises AssertionError on a real mismatch.
    `rows[b]` maps result row b to its query index in queries_np (default identity)."""
    g_ids, g_sc = np.asarray(g_ids), np.asarray(g_sc)
    B, k = o_ids.shape
    assert g_ids.shape == (B, k) and g_sc.shape == (B, k)
    strict = 0
    for b in range(B):
        qb = b if rows is None else int(rows[b])
        gi, oi = g_ids[b].tolist(), o_ids[b].tolist()
        # scores, rank by rank (padding -inf must match exactly)
        for j in range(k):
            if oi[j] < 0:
                assert gi[j] == -1 and np.isneginf(g_sc[b, j]), (b, j, gi, oi)
            else:
                assert abs(float(g_sc[b, j]) - o_sc64[b, j]) <= tol, (b, j, g_sc[b], o_sc64[b])
        if gi == oi:
            strict += 1
            continue
        valid = [i for i in oi if i >= 0]
        s_k = min(o_sc64[b, j] for j in range(k) if oi[j] >= 0)
        assert len(set(gi)) == len(gi) or -1 in gi, (b, gi)
        assert sum(i >= 0 for i in gi) == len(valid), (b, gi, oi)
        prev = np.inf
        for j, g in enumerate(gi):
            if g < 0:
                continue
            s = oracle.score(corpus_np, queries_np, qb, g, dtype)
            assert abs(s - float(g_sc[b, j])) <= tol, (b, g, s, g_sc[b, j])
            if g not in valid:
                assert s >= s_k - tol, (b, g, s, s_k)       # only a boundary near-tie may enter
            assert s <= prev + tol, (b, gi, oi)              # order may differ only inside a near-tie
            prev = s
        for j, o in enumerate(oi):
            if o >= 0 and o_sc64[b, j] > s_k + tol:
                assert o in gi, (b, o, gi, oi)               # clear members may not be lost
    return strict, B - strict, B


NEAR_TIE = 1e-6   # two fp64 oracle scores closer than this may be ordered the other way round in fp32


def walk(score_of, graph_row, N, entries, k, ef, max_expand=0):
    """The best-first search written once more, in Python, over a score function (used only to
    explain a trajectory that differs from the oracle's, never as the expected value of a test).
    Returns (top-k ids, n_dist, n_expand, {node: score})."""
    import bisect
    scored, L, expanded = {}, [], set()          # L: sorted list of (-score, id)
    n_expand = 0

    def offer(v):
        s = scored[v] = score_of(v)
        if s != s:
            return
        key = (-s, v)
        if len(L) == ef and not key < L[-1]:
            return
        bisect.insort(L, key)
        if len(L) > ef:
            L.pop()

    for e in entries:
        if 0 <= e < N and e not in scored:
            offer(int(e))
    while True:
        nxt = next((key for key in L if key[1] not in expanded), None)
        if nxt is None or (max_expand and n_expand >= max_expand):
            break
        expanded.add(nxt[1])
        n_expand += 1
        for v in graph_row(nxt[1]):
            v = int(v)
            if 0 <= v < N and v not in scored:
                offer(v)
    return [key[1] for key in L[:k]], len(scored), n_expand, scored


def explain_divergence(xn, gn, qn, b, name, entries, k, ef, o_ids, o_counters, g_ids, g_counters, tie=NEAR_TIE):
    """A GPU search whose counters (n_dist, n_expand) differ from the oracle's is accepted only if
    it is the oracle's search with the order of one or two pairs of near-tied nodes (fp64 scores
    closer than `tie`) reversed: the pairs are looked for among everything the oracle's walk scored,
    each is tried, and the walk that results must reproduce the GPU's ids and counters exactly.
    Returns [(node a, node b, |score gap|), ...]; raises AssertionError when no such pair exists."""
    import itertools
    N = xn.shape[0]
    memo = {}

    def base(v):
        if v not in memo:
            memo[v] = oracle.score(xn, qn, b, v, name)
        return memo[v]

    row = lambda v: gn[v]
    ids0, nd0, ne0, scored = walk(base, row, N, entries, k, ef)
    assert (ids0, nd0, ne0) == ([i for i in o_ids if i >= 0], o_counters[0], o_counters[1]), \
        ("the explaining walk must be the oracle's", b, ids0, nd0, ne0, o_ids, o_counters)
    order = sorted((s, v) for v, s in scored.items() if s == s)
    near = [(order[i][1], order[i + 1][1], order[i + 1][0] - order[i][0])
            for i in range(len(order) - 1) if order[i + 1][0] - order[i][0] < tie]
    want = ([i for i in g_ids if i >= 0], g_counters[0], g_counters[1])
    for n_swaps in (1, 2):
        for combo in itertools.combinations(near, n_swaps):
            swap = {}
            for a, c, _ in combo:
                swap[a], swap[c] = c, a
            if len(swap) != 2 * n_swaps:
                continue
            got = walk(lambda v: base(swap.get(v, v)), row, N, entries, k, ef)
            if (sorted(got[0]), got[1], got[2]) == (sorted(want[0]), want[1], want[2]):
                return [(a, c, gap) for a, c, gap in combo]
    raise AssertionError(f"query {b}: GPU counters {g_counters} differ from the oracle's {o_counters} and no "
                         f"near-tie (< {tie}) among {len(near)} candidate pairs explains it")


def compare_nonstall(gpu, o, xn, gn, qn, name, entry, k, ef, tau, window, max_off=None):
    """GPU (ids, scores, stats, ema) against the oracle's non-stall result (ids, sc, sc64, stats, ema).
    Queries with the same (early, scored, expansions) are compared list by list.  A query that
    left at another expansion made a borderline decision (the moving averages sit at tau): its
    list must be the oracle's list cut after the GPU's number of expansions.
    Returns (n_same, n_off)."""
    ids, sc, stats, ema = gpu
    o_ids, _, o_sc64, o_stats, o_ema = o
    B = qn.shape[0]
    same = [b for b in range(B) if stats[b].tolist() == o_stats[b].tolist()]
    off = [b for b in range(B) if stats[b].tolist() != o_stats[b].tolist()]
    if same:
        compare_topk(ids[same], sc[same], o_ids[same], o_sc64[same], xn, qn, dtype=name, rows=same)
        # RQ divides by (best - worst), which amplifies the last-bit differences of the scores
        assert np.allclose(ema[same], o_ema[same], rtol=5e-4, atol=5e-4)
    for b in off:
        if stats[b, 0] == 0 and o_stats[b, 0] == 0:
            # both stopped naturally after different walks: accepted only if reversing a near-tie of the
            # oracle's walk (two scored nodes closer than NEAR_TIE in fp64) gives exactly the GPU's walk
            compare_topk(ids[b:b + 1], sc[b:b + 1], o_ids[b:b + 1], o_sc64[b:b + 1], xn, qn, dtype=name, rows=[b])
            pairs = explain_divergence(xn, gn, qn, b, name, [entry], k, ef, o_ids[b].tolist(),
                                       (int(o_stats[b, 1]), int(o_stats[b, 2])), ids[b].tolist(),
                                       (int(stats[b, 1]), int(stats[b, 2])))
            print(f"  query {b}: walk differs from the oracle's at a near-tie: " +
                  ", ".join(f"nodes {a}/{c} gap {gap:.2e}" for a, c, gap in pairs), flush=True)
            continue
        cut = oracle.graph_search_nonstall(xn, gn, entry, qn[b:b + 1], k, ef, tau=np.inf, window=window,
                                           max_expand=int(stats[b, 2]), dtype=name)
        compare_topk(ids[b:b + 1], sc[b:b + 1], cut[0], cut[2], xn, qn, dtype=name, rows=[b])
        assert cut[3][0, 1] == stats[b, 1], (b, cut[3], stats[b])
        assert abs(float(cut[4][0]) - float(ema[b])) < 5e-4 * (1 + abs(float(ema[b])))
        assert abs(float(ema[b]) - tau) < 2e-3 or abs(float(o_ema[b]) - tau) < 2e-3, (b, ema[b], o_ema[b], tau)
    if max_off is None:
        max_off = max(1, B // 50)
    assert len(off) <= max_off, (len(off), B)
    return len(same), len(off)


def recall(approx_ids, exact_ids):
    return oracle.recall_at_k(np.asarray(approx_ids), np.asarray(exact_ids))
