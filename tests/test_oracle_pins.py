"""Pins for the CPU oracle: it is checked against things other than itself —
closed forms, library routines on special cases, a hand trace, a second
set-based formulation of the beam search, and invariants — chosen so that a
dropped term, a wrong sign or index, a transposed operand or a wrong tie rule
fails at least one of them.  No GPU, no product code."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def unit_rows(n, d, dtype=np.float32):
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(dtype)


# ---------------------------------------------------------------- storage decoding

def test_half_decode_all_bit_patterns():
    """Every fp16 bit pattern, scored against q = [1], must decode exactly as numpy does."""
    bits = np.arange(65536, dtype=np.uint16)
    corpus = bits.view(np.float16).reshape(-1, 1)
    q = np.array([[1.0]], np.float16)
    want = corpus.astype(np.float64)[:, 0]
    for row in list(range(0, 65536, 257)) + [0, 1, 0x3ff, 0x400, 0x7bff, 0x8000, 0x8001, 0xfbff, 0x3c00]:
        if np.isnan(want[row]) or np.isinf(want[row]):
            continue
        assert oracle.score(corpus, q, 0, row) == want[row], hex(row)


def test_bf16_decode_matches_torch():
    t = torch.randn(4096).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16).reshape(-1, 1)
    q = torch.ones(1, 1, dtype=torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    want = t.double().numpy()
    for row in range(0, 4096, 37):
        assert oracle.score(bits, q, 0, row, dtype="bf16") == want[row]


def test_accumulates_in_double():
    """1 + 2^-30 - 1 is 2^-30 in double and 0 in fp32."""
    corpus = np.array([[1.0, 2.0 ** -30, -1.0]], np.float32)
    q = np.ones((1, 3), np.float32)
    assert oracle.score(corpus, q, 0, 0) == 2.0 ** -30
    _, _, s64 = oracle.flat_search(corpus, q, 1)
    assert s64[0, 0] == 2.0 ** -30


# ---------------------------------------------------------------- exact retrieval

def test_flat_closed_form_basis_corpus():
    """Corpus = signed, scaled basis vectors: score(n) = c_n * q[perm[n]], so the
    exact top-k is known without any dot product.  Catches transposed operands,
    wrong row strides and a wrong sign of the order."""
    d = 24
    perm = rng.permutation(d)
    coef = rng.uniform(0.5, 2.0, d).astype(np.float32) * rng.choice([-1.0, 1.0], d).astype(np.float32)
    corpus = np.zeros((d, d), np.float32)
    corpus[np.arange(d), perm] = coef
    q = rng.standard_normal((5, d)).astype(np.float32)
    ids, sc, sc64 = oracle.flat_search(corpus, q, 6)
    for b in range(5):
        closed = coef.astype(np.float64) * q[b, perm].astype(np.float64)
        want = sorted(range(d), key=lambda n: (-closed[n], n))[:6]
        assert ids[b].tolist() == want
        assert np.array_equal(sc64[b], closed[want])
        assert np.array_equal(sc[b], closed[want].astype(np.float32))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_flat_matches_numpy_matmul_lexsort(dtype):
    corpus = unit_rows(700, 40, dtype)
    q = unit_rows(9, 40, dtype)
    k = 12
    ids, sc, sc64 = oracle.flat_search(corpus, q, k)
    S = q.astype(np.float64) @ corpus.astype(np.float64).T
    for b in range(q.shape[0]):
        order = np.lexsort((np.arange(700), -S[b]))[:k]
        assert ids[b].tolist() == order.tolist()
        np.testing.assert_allclose(sc64[b], S[b, order], rtol=0, atol=1e-14)
        assert np.all(np.diff(sc64[b]) <= 0)
    # k = 1 is the arg-max
    ids1, _, _ = oracle.flat_search(corpus, q, 1)
    assert ids1[:, 0].tolist() == np.argmax(S, axis=1).tolist()
    # k = N returns a permutation of all rows
    idsN, _, _ = oracle.flat_search(corpus, q[:2], 700)
    assert sorted(idsN[0].tolist()) == list(range(700))


def test_flat_ties_go_to_lower_id():
    corpus = unit_rows(50, 16)
    corpus[37] = corpus[5]
    corpus[44] = corpus[5]
    q = corpus[5:6].copy()
    ids, _, sc64 = oracle.flat_search(corpus, q, 4)
    assert ids[0, :3].tolist() == [5, 37, 44]
    assert sc64[0, 0] == sc64[0, 1] == sc64[0, 2]


def test_flat_continuation_enumerates_the_corpus_in_order():
    """Pages of k rows, each started after the last pair of the one before, concatenate to the one answer
    with all rows; tied scores are split between pages by id."""
    n, d = 57, 6
    corpus = unit_rows(n, d)
    corpus[10] = corpus[3]
    corpus[41] = corpus[3]                      # three identical rows: a tie that a page boundary will cut
    q = unit_rows(4, d)
    full_ids, _, full_sc = oracle.flat_search(corpus, q, n)
    for k in (1, 5, 16):
        after, got = None, []
        for _ in range((n + k - 1) // k):
            ids, _, sc = oracle.flat_search(corpus, q, k, after=after)
            got.append(ids)
            last = np.array([[j for j in range(k) if ids[b, j] >= 0][-1] for b in range(4)])
            after = (sc[np.arange(4), last], ids[np.arange(4), last])
        got = np.concatenate(got, 1)
        assert np.array_equal(got[:, :n], full_ids)
        assert (got[:, n:] == -1).all()
    # nothing excluded: a NaN boundary; everything excluded: a boundary after the last row
    ids, _, _ = oracle.flat_search(corpus, q, 3, after=(np.full(4, np.nan), np.zeros(4, np.int32)))
    assert np.array_equal(ids, full_ids[:, :3])
    ids, sc, _ = oracle.flat_search(corpus, q, 3, after=(full_sc[:, -1], full_ids[:, -1]))
    assert (ids == -1).all() and np.isneginf(sc).all()


def test_flat_rejects_bad_arguments():
    corpus = unit_rows(10, 8)
    with pytest.raises(ValueError):
        oracle.flat_search(corpus, corpus[:2], 11)
    with pytest.raises(ValueError):
        oracle.flat_search(corpus, corpus[:2], 0)


# ---------------------------------------------------------------- graph retrieval

def read_trace():
    values, cases, exact = None, [], None
    for line in open(os.path.join(GOLDEN, "path_graph_trace.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("values"):
            values = [float(t) for t in line.split()[1:]]
        elif line.startswith("case"):
            a, b, c = line[4:].split("|")
            ef, k = (int(t) for t in a.split())
            nd, ne = (int(t) for t in c.split())
            cases.append((ef, k, [int(t) for t in b.split()], nd, ne))
        elif line.startswith("nonstall"):
            continue
        elif line.startswith("exact3"):
            exact = [int(t) for t in line.split("|")[1].split()]
    return values, cases, exact


def path_graph(n):
    g = np.full((n, 2), -1, np.int32)
    g[1:, 0] = np.arange(n - 1)
    g[:-1, 1] = np.arange(1, n)
    return g


def test_graph_hand_trace():
    values, cases, exact = read_trace()
    corpus = np.array(values, np.float32).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    g = path_graph(len(values))
    for ef, k, want_ids, want_nd, want_ne in cases:
        ids, sc, _, nd, ne = oracle.graph_search(corpus, g, 0, q, k, ef)
        assert ids[0].tolist() == want_ids, (ef, ids)
        assert (int(nd[0]), int(ne[0])) == (want_nd, want_ne), ef
        assert sc[0].tolist() == [np.float32(values[i]) for i in want_ids]
    ids, _, _ = oracle.flat_search(corpus, q, 3)
    assert ids[0].tolist() == exact
    g_ids = oracle.graph_search(corpus, g, 0, q, 3, 3)[0]
    assert oracle.recall_at_k(g_ids, ids) == pytest.approx(2 / 3)


def beam_search_by_sets(S, graph, entry, k, ef):
    """Second formulation: after every scored node the list is *recomputed* as the
    best ef of everything scored so far; expanded nodes are a set of ids."""
    N, R = graph.shape
    key = lambda v: (-S[v], v)
    seen = {entry}
    expanded = set()
    n_expand = 0
    while True:
        L = sorted(seen, key=key)[:ef]
        todo = [v for v in L if v not in expanded]
        if not todo:
            break
        p = todo[0]
        expanded.add(p)
        n_expand += 1
        for v in graph[p]:
            v = int(v)
            if 0 <= v < N:
                seen.add(v)
    L = sorted(seen, key=key)[:ef]
    return L[:k], len(seen), n_expand


def random_graph(n, R, p_empty=0.1):
    g = rng.integers(0, n, size=(n, R)).astype(np.int32)
    g[rng.random((n, R)) < p_empty] = -1
    return g


@pytest.mark.parametrize("ef", [1, 2, 5, 16, 64])
def test_graph_matches_set_formulation(ef):
    n, d, R = 48, 12, 4
    corpus = unit_rows(n, d)
    q = unit_rows(6, d)
    g = random_graph(n, R)
    g[3, 0] = n + 5          # out-of-range id must be skipped
    g[7, 1] = 7              # self loop
    g[9, 2] = g[9, 3]        # duplicate in a row
    S = q.astype(np.float64) @ corpus.astype(np.float64).T
    k = min(ef, 3)
    ids, _, sc64, nd, ne = oracle.graph_search(corpus, g, 11, q, k, ef)
    for b in range(q.shape[0]):
        want, n_seen, n_exp = beam_search_by_sets(S[b], g, 11, k, ef)
        got = [i for i in ids[b].tolist() if i >= 0]
        assert got == want, (b, ef)
        assert int(nd[b]) == n_seen and int(ne[b]) == n_exp
        assert int(nd[b]) <= 1 + R * int(ne[b])
        np.testing.assert_allclose(sc64[b, :len(got)], S[b, got], atol=1e-14)


def connected_graph(n, R):
    g = random_graph(n, R)
    i = np.arange(n, dtype=np.int32)
    return np.concatenate([g, ((i + 1) % n)[:, None], ((i - 1) % n)[:, None]], 1).astype(np.int32)


def test_graph_with_ef_at_least_n_on_connected_graph_is_exact():
    n, d = 300, 24
    corpus = unit_rows(n, d, np.float16)
    q = unit_rows(10, d, np.float16)
    g = connected_graph(n, 6)
    f_ids, f_sc, f_sc64 = oracle.flat_search(corpus, q, 10)
    for ef in (n, n + 17):
        ids, sc, sc64, nd, ne = oracle.graph_search(corpus, g, 123, q, 10, ef)
        assert np.array_equal(ids, f_ids)
        assert np.array_equal(sc64, f_sc64)
        assert np.all(nd == n) and np.all(ne == n)


def test_graph_complete_graph_any_ef_is_exact():
    n, d = 40, 8
    corpus = unit_rows(n, d)
    q = unit_rows(7, d)
    g = np.array([[j for j in range(n) if j != i] for i in range(n)], np.int32)
    f_ids, _, _ = oracle.flat_search(corpus, q, 5)
    for ef in (5, 9, 40):
        ids = oracle.graph_search(corpus, g, 0, q, 5, ef)[0]
        assert np.array_equal(ids, f_ids)


def test_graph_invariants_and_padding():
    n, d, R = 200, 16, 5
    corpus = unit_rows(n, d)
    q = unit_rows(12, d)
    g = random_graph(n, R, 0.2)
    # two islands: nodes < 60 only point below 60, the rest only at or above 60
    g[:60] = np.where(g[:60] >= 0, g[:60] % 60, -1)
    g[60:] = np.where(g[60:] >= 0, 60 + g[60:] % (n - 60), -1)
    f_ids, _, f64 = oracle.flat_search(corpus, q, 8)
    ids, sc, sc64, nd, ne = oracle.graph_search(corpus, g, 5, q, 8, 32)
    for b in range(q.shape[0]):
        got = [i for i in ids[b].tolist() if i >= 0]
        assert len(set(got)) == len(got)
        assert all(i < 60 for i in got)                       # stays in the entry's island
        assert np.all(np.diff(sc64[b, :len(got)]) <= 0)
        assert np.all(sc64[b, :len(got)] <= f64[b, :len(got)] + 1e-15)   # rank-wise bound
    # a sink entry: only the entry itself is reachable, the rest is padding
    g2 = g.copy()
    g2[5] = -1
    ids, sc, _, nd, ne = oracle.graph_search(corpus, g2, 5, q[:2], 4, 8)
    assert ids.tolist() == [[5, -1, -1, -1]] * 2
    assert np.all(np.isneginf(sc[:, 1:])) and np.all(nd == 1) and np.all(ne == 1)


def test_graph_tie_rule_prefers_lower_id():
    """Two identical vectors: the lower id is listed first and expanded first."""
    corpus = unit_rows(6, 4)
    corpus[4] = corpus[2]
    q = corpus[2:3].copy()
    g = np.array([[4, 2], [-1, -1], [1, -1], [-1, -1], [3, -1], [-1, -1]], np.int32)
    # from 0: scores 4 then 2 (equal scores). ef=2 keeps both, order must be [2, 4].
    ids, _, _, nd, ne = oracle.graph_search(corpus, g, 0, q, 2, 2)
    assert ids[0].tolist() == [2, 4]
    # with ef = 1 node 4 is listed first (0 dropped), then 2 is scored with an equal
    # score and the lower id, so it precedes 4 and replaces it
    ids, _, _, _, _ = oracle.graph_search(corpus, g, 0, q, 1, 1)
    assert ids[0].tolist() == [2]


def test_graph_rejects_bad_arguments():
    corpus = unit_rows(10, 8)
    g = random_graph(10, 3)
    with pytest.raises(ValueError):
        oracle.graph_search(corpus, g, 0, corpus[:1], 4, 3)      # ef < k
    with pytest.raises(ValueError):
        oracle.graph_search(corpus, g, 10, corpus[:1], 1, 4)     # entry out of range


def test_recall_definition():
    exact = np.array([[1, 2, 3], [4, 5, 6]], np.int32)
    approx = np.array([[3, 9, 1], [-1, -1, 4]], np.int32)
    assert oracle.recall_at_k(approx, exact) == pytest.approx(3 / 6)


# ---------------------------------------------------------------- maturity (non-stall) exit

def read_nonstall_trace():
    out = []
    for line in open(os.path.join(GOLDEN, "path_graph_trace.txt")):
        if line.startswith("nonstall"):
            a, b, c, e = line[len("nonstall"):].split("|")
            w, tau, rf = a.split()
            out.append((int(w), float(tau), int(rf), [int(t) for t in b.split()], [int(t) for t in c.split()], float(e)))
    return out


def test_nonstall_hand_trace():
    values, _, _ = read_trace()
    corpus = np.array(values, np.float32).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    g = path_graph(len(values))
    cases = read_nonstall_trace()
    assert len(cases) == 5
    for w, tau, rf, want_ids, want_stats, want_ema in cases:
        ids, _, _, stats, ema = oracle.graph_search_nonstall(corpus, g, 0, q, 3, 3, tau=tau, window=w, ready_from=rf)
        assert ids[0].tolist() == want_ids, (w, tau, rf)
        assert stats[0].tolist() == want_stats, (w, tau, rf)
        assert ema[0] == pytest.approx(want_ema, abs=2e-6)


def test_nonstall_constant_rq_closed_form():
    """Path graph, scores 1, 0, 0, 0, ...: from the second expansion on every new node has
    RQ = (1 - 0) / (1 - 0) = 1, so after n samples EMA = 1 - (1 - alpha)^n and the exit
    comes at the first n with EMA > tau: n = floor(ln(1 - tau) / ln(1 - alpha)) + 1."""
    n = 1500
    corpus = np.zeros((n, 1), np.float32)
    corpus[0] = 1.0
    q = np.ones((1, 1), np.float32)
    g = path_graph(n)
    for window, tau in ((500, 0.9), (100, 0.5), (20, 0.97)):
        alpha = 2.0 / (window + 1)
        n_samples = int(np.floor(np.log(1 - tau) / np.log(1 - alpha))) + 1
        assert abs((1 - (1 - alpha) ** n_samples) - tau) > 1e-4          # not a borderline decision
        assert abs((1 - (1 - alpha) ** (n_samples - 1)) - tau) > 1e-4
        ids, _, _, stats, ema = oracle.graph_search_nonstall(corpus, g, 0, q, 3, n, tau=tau, window=window)
        early, nd, ne = stats[0].tolist()
        assert early == 1
        assert ne == n_samples + 1                    # the first expansion yields no sample
        assert nd == ne + 1
        assert ema[0] == pytest.approx(1 - (1 - alpha) ** n_samples, abs=1e-4)
        assert ids[0].tolist() == [0, 1, 2]


def nonstall_by_sets(S, graph, entry, ef, tau, alpha, ready_from):
    """Second formulation in double precision: the list is recomputed as the best ef of all
    scored nodes; returns (early, n_dist, n_expand, min |EMA - tau| seen at a test)."""
    N = len(S)
    key = lambda v: (-S[v], v)
    scored, expanded, ema, margin = {entry}, set(), 0.0, np.inf
    while True:
        L = sorted(scored, key=key)[:ef]
        todo = [v for v in L if v not in expanded]
        if not todo:
            return 0, len(scored), len(expanded), margin
        p = todo[0]
        expanded.add(p)
        best, worst = S[L[0]], S[L[-1]]
        for v in graph[p]:
            if 0 <= v < N and v not in scored:
                scored.add(int(v))
                if len(L) >= 2 and best != worst:
                    ema += alpha * ((best - S[v]) / (best - worst) - ema)
        margin = min(margin, abs(ema - tau))
        if ema > tau and len(expanded) >= ready_from:
            return 1, len(scored), len(expanded), margin


@pytest.mark.parametrize("ef,window,tau,ready_from", [(8, 10, 0.7, 0), (16, 30, 0.8, 0), (16, 30, 0.8, 12), (32, 60, 0.9, 0), (4, 5, 0.5, 3)])
def test_nonstall_matches_set_formulation(ef, window, tau, ready_from):
    n, R = 400, 6
    x = unit_rows(n, 12)
    g = random_graph(n, R)
    q = unit_rows(6, 12)
    S = x.astype(np.float64) @ q.astype(np.float64).T
    _, _, _, stats, _ = oracle.graph_search_nonstall(x, g, 0, q, 3, ef, tau=tau, window=window, ready_from=ready_from)
    checked = 0
    for b in range(q.shape[0]):
        early, nd, ne, margin = nonstall_by_sets(S[:, b], g, 0, ef, tau, 2.0 / (window + 1), ready_from)
        if margin < 1e-4:         # binary32 vs double could decide differently: not a pin
            continue
        assert stats[b].tolist() == [early, nd, ne], b
        checked += 1
    assert checked >= 4


def test_nonstall_never_triggered_equals_natural_stop():
    n = 600
    x = unit_rows(n, 16)
    g = random_graph(n, 8)
    q = unit_rows(5, 16)
    ref = oracle.graph_search(x, g, 0, q, 4, 24)
    for kw in (dict(tau=np.inf), dict(tau=0.1, ready_from=1 << 40)):
        ids, sc, sc64, stats, _ = oracle.graph_search_nonstall(x, g, 0, q, 4, 24, window=7, **kw)
        assert np.array_equal(ids, ref[0]) and np.array_equal(sc64, ref[2])
        assert np.array_equal(stats[:, 0], np.zeros(5, np.int32))
        assert np.array_equal(stats[:, 1], ref[3]) and np.array_equal(stats[:, 2], ref[4])


def test_nonstall_exit_returns_the_state_of_the_full_search_at_that_point():
    """An early exit only cuts the search short: its result is what the natural search
    holds after the same number of expansions, and it never expands more."""
    n = 800
    x = unit_rows(n, 16)
    g = random_graph(n, 8)
    q = unit_rows(8, 16)
    nat = oracle.graph_search(x, g, 0, q, 3, 32)
    ids, _, sc64, stats, _ = oracle.graph_search_nonstall(x, g, 0, q, 3, 32, tau=0.6, window=15)
    assert stats[:, 0].sum() >= 4
    for b in range(8):
        assert stats[b, 2] <= nat[4][b]
        cut = oracle.graph_search_nonstall(x, g, 0, q[b:b + 1], 3, 32, tau=np.inf, max_expand=int(stats[b, 2]))
        assert np.array_equal(cut[0][0], ids[b]) and np.array_equal(cut[2][0], sc64[b])
        assert cut[3][0, 1] == stats[b, 1]



# ---------------------------------------------------------------- several entry nodes per query

def read_multi_trace():
    out = []
    for line in open(os.path.join(GOLDEN, "path_graph_trace.txt")):
        if line.startswith("multi"):
            a, e, b, c = line[len("multi"):].split("|")
            ef, k = (int(t) for t in a.split())
            out.append((ef, k, [int(t) for t in e.split()], [int(t) for t in b.split()], [int(t) for t in c.split()]))
    return out


def test_multi_entry_hand_trace():
    values, _, _ = read_trace()
    corpus = np.array(values, np.float32).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    g = path_graph(len(values))
    cases = read_multi_trace()
    assert len(cases) == 3
    for ef, k, entries, want_ids, (want_nd, want_ne) in cases:
        ids, _, _, nd, ne = oracle.graph_search(corpus, g, 0, q, k, ef, entries=np.array([entries], np.int32))
        assert ids[0].tolist() == want_ids, entries
        assert (int(nd[0]), int(ne[0])) == (want_nd, want_ne), entries
        # the maturity variant with a threshold that is never reached runs the same search
        ids2, _, _, stats, _ = oracle.graph_search_nonstall(corpus, g, 0, q, k, ef, tau=np.inf,
                                                            entries=np.array([entries], np.int32))
        assert ids2[0].tolist() == want_ids and stats[0].tolist() == [0, want_nd, want_ne]


def beam_search_by_sets_multi(S, graph, entries, k, ef):
    """The set formulation above, started from several nodes."""
    N = graph.shape[0]
    key = lambda v: (-S[v], v)
    seen = {int(e) for e in entries if 0 <= e < N}
    expanded, n_expand = set(), 0
    while True:
        L = sorted(seen, key=key)[:ef]
        todo = [v for v in L if v not in expanded]
        if not todo:
            return L[:k], len(seen), n_expand
        expanded.add(todo[0])
        n_expand += 1
        seen |= {int(v) for v in graph[todo[0]] if 0 <= v < N}


@pytest.mark.parametrize("ef,E", [(1, 3), (4, 2), (4, 9), (16, 5), (64, 32)])
def test_multi_entry_matches_set_formulation(ef, E):
    n, d, R = 60, 12, 4
    corpus = unit_rows(n, d)
    q = unit_rows(5, d)
    g = random_graph(n, R)
    S = q.astype(np.float64) @ corpus.astype(np.float64).T
    entries = rng.integers(-2, n + 2, size=(5, E)).astype(np.int32)      # some out of range, some repeated
    entries[0, :] = entries[0, 0]
    k = min(ef, 3)
    ids, _, _, nd, ne = oracle.graph_search(corpus, g, 0, q, k, ef, entries=entries)
    for b in range(5):
        want, n_seen, n_exp = beam_search_by_sets_multi(S[b], g, entries[b], k, ef)
        assert [i for i in ids[b].tolist() if i >= 0] == want, (b, ef)
        assert (int(nd[b]), int(ne[b])) == (n_seen, n_exp)


def test_multi_entry_special_cases():
    n, d = 120, 16
    corpus = unit_rows(n, d, np.float16)
    q = unit_rows(6, d, np.float16)
    g = random_graph(n, 5)
    # one entry per query given as a list is the single-entry search
    one = oracle.graph_search(corpus, g, 17, q, 4, 12)
    lst = oracle.graph_search(corpus, g, 0, q, 4, 12, entries=np.full((6, 1), 17, np.int32))
    for a, b in zip(one, lst):
        assert np.array_equal(a, b)
    # every node an entry and ef = N: the list holds the whole corpus, i.e. the exact answer,
    # whatever the graph
    f_ids, _, f64 = oracle.flat_search(corpus, q, 7)
    allnodes = np.tile(np.arange(n, dtype=np.int32), (6, 1))
    ids, _, sc64, nd, _ = oracle.graph_search(corpus, g, 0, q, 7, n, entries=allnodes)
    assert np.array_equal(ids, f_ids) and np.array_equal(sc64, f64) and np.all(nd == n)
    # no valid entry: nothing is reachable
    ids, sc, _, nd, ne = oracle.graph_search(corpus, g, 0, q, 3, 8, entries=np.full((6, 2), -1, np.int32))
    assert np.all(ids == -1) and np.all(np.isneginf(sc)) and np.all(nd == 0) and np.all(ne == 0)


def test_nan_scores_are_never_listed():
    values, _, _ = read_trace()
    corpus = np.array(values, np.float32).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    g = path_graph(len(values))
    bad = corpus.copy()
    bad[2] = np.nan                      # the walk 0 -> 1 -> 2 -> 3 cannot pass node 2
    f_ids, f_sc, _ = oracle.flat_search(bad, q, 8)
    assert f_ids[0].tolist() == [3, 7, 5, 1, 4, 0, 6, -1] and np.isneginf(f_sc[0, 7])   # values .9 .9 .5 .3 .3 .1 .05
    ids, sc, _, nd, ne = oracle.graph_search(bad, g, 0, q, 3, 3)
    assert ids[0].tolist() == [1, 0, -1] and np.isneginf(sc[0, 2])
    assert (int(nd[0]), int(ne[0])) == (3, 2)                # node 2 is scored and counted, not listed
    ids, sc, _, nd, ne = oracle.graph_search(bad, g, 2, q, 2, 3)
    assert ids[0].tolist() == [-1, -1] and (int(nd[0]), int(ne[0])) == (1, 0)    # a NaN entry: nothing to expand
    for form in ("node", "expansion"):
        ids, _, _, stats, ema = oracle.graph_search_nonstall(bad, g, 0, q, 3, 3, tau=np.inf, form=form)
        assert ids[0].tolist() == [1, 0, -1] and stats[0].tolist() == [0, 3, 2] and ema[0] == 0.0


# ---------------------------------------------------------------- the two forms of RQ's best / worst

def read_star_trace():
    values, rows, natural, cases = None, [], None, []
    for line in open(os.path.join(GOLDEN, "star_graph_trace.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("values"):
            values = [float(t) for t in line.split()[1:]]
        elif line.startswith("row"):
            rows.append([int(t) for t in line.split()[1:]])
        elif line.startswith("natural"):
            _, b, c = line.split("|")
            natural = ([int(t) for t in b.split()], [int(t) for t in c.split()])
        elif line.startswith("nonstall"):
            a, b, c, e = line[len("nonstall"):].split("|")
            form, w, tau, rf = a.split()
            cases.append((form, int(w), float(tau), int(rf), [int(t) for t in b.split()], [int(t) for t in c.split()], float(e)))
    return values, np.array(rows, np.int32), natural, cases


def test_rq_forms_hand_trace():
    values, g, (nat_ids, (nat_nd, nat_ne)), cases = read_star_trace()
    corpus = np.array(values, np.float32).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    ids, _, _, nd, ne = oracle.graph_search(corpus, g, 0, q, 3, 3)
    assert ids[0].tolist() == nat_ids and (int(nd[0]), int(ne[0])) == (nat_nd, nat_ne)
    assert len(cases) == 8 and {c[0] for c in cases} == {"node", "expansion"}
    for form, w, tau, rf, want_ids, want_stats, want_ema in cases:
        ids, _, _, stats, ema = oracle.graph_search_nonstall(corpus, g, 0, q, 3, 3, tau=tau, window=w, form=form,
                                                            ready_from=rf)
        assert ids[0].tolist() == want_ids, (form, tau, rf)
        assert stats[0].tolist() == want_stats, (form, tau, rf)
        assert ema[0] == pytest.approx(want_ema, abs=5e-6), (form, tau, rf)


def nonstall_per_node_by_sets(S, graph, entry, ef, tau, alpha, ready_from):
    """Per-node form, second formulation in double precision: the list is recomputed as the best ef
    of all scored nodes before every single node is scored."""
    N = len(S)
    key = lambda v: (-S[v], v)
    scored, expanded, ema, margin = {entry}, set(), 0.0, np.inf
    while True:
        L = sorted(scored, key=key)[:ef]
        todo = [v for v in L if v not in expanded]
        if not todo:
            return 0, len(scored), len(expanded), margin, ema
        p = todo[0]
        expanded.add(p)
        for v in graph[p]:
            if 0 <= v < N and v not in scored:
                L = sorted(scored, key=key)[:ef]
                best, worst = S[L[0]], S[L[-1]]
                scored.add(int(v))
                if len(L) >= 2 and best != worst:
                    ema += alpha * ((best - S[v]) / (best - worst) - ema)
        margin = min(margin, abs(ema - tau))
        if ema > tau and len(expanded) >= ready_from:
            return 1, len(scored), len(expanded), margin, ema


@pytest.mark.parametrize("ef,window,tau,ready_from", [(8, 10, 0.7, 0), (16, 30, 0.8, 0), (16, 30, 0.8, 12), (32, 60, 0.9, 0), (4, 5, 0.5, 3)])
def test_nonstall_per_node_matches_set_formulation(ef, window, tau, ready_from):
    n, R = 400, 6
    x = unit_rows(n, 12)
    g = random_graph(n, R)
    q = unit_rows(6, 12)
    S = x.astype(np.float64) @ q.astype(np.float64).T
    _, _, _, stats, ema = oracle.graph_search_nonstall(x, g, 0, q, 3, ef, tau=tau, window=window, form="node",
                                                       ready_from=ready_from)
    checked = 0
    for b in range(q.shape[0]):
        early, nd, ne, margin, want_ema = nonstall_per_node_by_sets(S[:, b], g, 0, ef, tau, 2.0 / (window + 1), ready_from)
        if margin < 1e-9:
            continue
        assert stats[b].tolist() == [early, nd, ne], b
        assert ema[b] == pytest.approx(want_ema, rel=1e-5, abs=1e-6)
        checked += 1
    assert checked >= 5


def test_rq_forms_agree_when_one_node_is_scored_per_expansion():
    """On a path graph entered at its end every expansion scores at most one new node, so the list "when the node is
    scored" is the list "when the expansion starts": both forms give the same exits and averages."""
    n = 300
    x = unit_rows(n, 8)
    q = unit_rows(4, 8)
    g = path_graph(n)
    for tau in (0.3, 0.6, 0.9):
        a = oracle.graph_search_nonstall(x, g, 0, q, 3, 16, tau=tau, window=12, form="node")
        b = oracle.graph_search_nonstall(x, g, 0, q, 3, 16, tau=tau, window=12, form="expansion")
        close = np.abs(a[4] - tau) < 1e-4
        assert np.array_equal(a[3][~close], b[3][~close])
        np.testing.assert_allclose(a[4][~close], b[4][~close], rtol=2e-4, atol=2e-5)


def test_rq_forms_differ_measurably_on_a_clustered_workload():
    """How far the per-expansion form (what a search that scores a node's neighbours together computes)
    is from the per-node form (Section 3.3 read for a one-node-at-a-time search), on a scaled
    clustered workload: both must stop early for a comparable share of the queries and return
    lists of comparable recall; the numbers at full size are reported by the benchmark."""
    from paper_2505_12065_amd import synth
    c = synth.make_corpus(20_000, 64, 24, seed=5, dtype=torch_f16())
    qn = synth.make_queries(c, 48, noise_std=0.05 / 8).numpy()
    xn = c.x.numpy()
    g = synth.with_reverse_edges(synth.knn_graph(c.x, 16), c.x).numpy()
    exact = oracle.flat_search(xn, qn, 3)[0]
    out = {}
    for form in ("node", "expansion"):
        ids, _, _, stats, _ = oracle.graph_search_nonstall(xn, g, 0, qn, 3, 64, tau=0.9, window=50, form=form)
        out[form] = (stats, oracle.recall_at_k(ids, exact))
    (sa, ra), (sb, rb) = out["node"], out["expansion"]
    differ = int((sa[:, 2] != sb[:, 2]).sum())
    print(f"RQ forms: early node={sa[:, 0].mean():.2f} expansion={sb[:, 0].mean():.2f}; "
          f"{differ}/48 leave at another expansion; mean expansions {sa[:, 2].mean():.1f} vs {sb[:, 2].mean():.1f}; "
          f"recall@3 {ra:.3f} vs {rb:.3f}")
    assert abs(sa[:, 0].mean() - sb[:, 0].mean()) <= 0.25
    assert abs(ra - rb) <= 0.15


def torch_f16():
    import torch
    return torch.float16


# ---------------------------------------------------------------- priority levels (Section 3.2, Eq. 1-2)

def test_priority_hand_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "priority_levels.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = v
    G = int(rows["G"][0])
    level, order = oracle.priority_order([int(t) for t in rows["R"]], [float(t) for t in rows["W"]],
                                         [int(t) for t in rows["C"]], [float(t) for t in rows["Wcur"]], G)
    assert level.tolist() == [int(t) for t in rows["level"]]
    assert order.tolist() == [int(t) for t in rows["order"]]


def test_priority_single_metric_closed_form():
    """With one metric varying, level = ceil(G (M - min) / range) - 1 for M > min (exact integer
    arithmetic; values that sit exactly on a threshold are left out)."""
    n, G = 500, 7
    R = rng.integers(3, 1000, n).astype(np.int32)
    R[0], R[1] = 3, 999
    mn, mx = int(R.min()), int(R.max())
    const = np.full(n, 4, np.int32)
    zeros = np.zeros(n)
    for which in range(3):
        args = [const, zeros + 2.5, const]
        args[which] = R if which != 1 else R.astype(np.float64)
        level, _ = oracle.priority_order(args[0], args[1], args[2], zeros, G)
        for i in range(n):
            num = G * (int(R[i]) - mn)
            if num % (mx - mn) == 0 and num != 0:
                continue
            want = 0 if num == 0 else -(-num // (mx - mn)) - 1
            assert level[i] == want, (which, i, R[i])
    assert level[1] == G - 1


def test_priority_nan_queueing_time_is_the_shortest_wait():
    R = np.array([1, 1, 1, 9, 1], np.int32)
    C = np.array([5, 5, 5, 5, 5], np.int32)
    W = np.array([1.0, 1.0, 1.0, 1.0, 1.0])
    Wcur = np.array([2.0, np.nan, 3.0, np.nan, np.nan])
    level, order = oracle.priority_order(R, W, C, Wcur, 6)
    assert level.tolist() == [0, 0, 0, 5, 0]
    assert order.tolist() == [3, 2, 0, 1, 4]      # top level first; then 3.0, 2.0, and the NaNs in index order


def test_priority_invariants_and_order():
    n, G = 300, 6
    R = rng.integers(0, 9, n).astype(np.int32)
    C = rng.integers(100, 5000, n).astype(np.int32)
    W = rng.random(n) * 30
    Wcur = np.round(rng.random(n) * 4, 1)                   # many equal queueing times
    level, order = oracle.priority_order(R, W, C, Wcur, G)
    assert level.min() >= 0 and level.max() == G - 1
    assert sorted(order.tolist()) == list(range(n))
    assert order.tolist() == sorted(range(n), key=lambda i: (-int(level[i]), -Wcur[i], i))
    for m in (R, W, C):                                      # the largest value of any metric is top level
        assert level[int(np.argmax(m))] == G - 1
    # shifting a metric, or scaling the waiting times by a power of two, changes nothing
    l2, o2 = oracle.priority_order(R + 5, W * 4 + 16, C + 1000, Wcur * 2, G)
    assert np.array_equal(l2, level) and np.array_equal(o2, order)
    # relabelling the requests relabels the result
    perm = rng.permutation(n)
    l3, _ = oracle.priority_order(R[perm], W[perm], C[perm], Wcur[perm], G)
    assert np.array_equal(l3, level[perm])
    # a request whose three metrics are all at the minimum is at the base level
    R[7], W[7], C[7] = R.min(), W.min(), C.min()
    assert oracle.priority_order(R, W, C, Wcur, G)[0][7] == 0
    # every metric constant: everybody at level 0, order by queueing time only
    one = np.ones(n, np.int32)
    l4, o4 = oracle.priority_order(one, np.ones(n), one, Wcur, G)
    assert not l4.any() and o4.tolist() == sorted(range(n), key=lambda i: (-Wcur[i], i))
