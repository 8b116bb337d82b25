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


def recall(approx_ids, exact_ids):
    return oracle.recall_at_k(np.asarray(approx_ids), np.asarray(exact_ids))
