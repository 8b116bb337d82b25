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
            # both stopped naturally: a near-tie ordered by fp32 rounding sent the two searches through
            # slightly different expansions; the lists must still agree under the near-tie rule
            compare_topk(ids[b:b + 1], sc[b:b + 1], o_ids[b:b + 1], o_sc64[b:b + 1], xn, qn, dtype=name, rows=[b])
            assert abs(int(stats[b, 1]) - int(o_stats[b, 1])) <= max(64, o_stats[b, 1] // 20), (b, stats[b], o_stats[b])
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
