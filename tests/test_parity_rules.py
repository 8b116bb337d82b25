"""The comparison rules of tests/parity.py checked on the CPU, with the deviations planted on the
oracle's side: a result that differs from the oracle's is accepted only for the stated reasons."""
import numpy as np
import pytest

import oracle
from parity import compare_topk, explain_divergence, walk

rng = np.random.default_rng(11)


def chain_with_a_fork(gap):
    """d = 1, query [1]: node 0 leads to nodes 1 and 2 whose scores differ by `gap`; each of them
    leads into a branch of its own, and with ef = 1 only the better one is expanded."""
    n = 40
    values = np.linspace(0.30, 0.10, n).astype(np.float64)
    values[0] = 0.05
    values[1] = 0.5
    values[2] = 0.5 - gap
    g = np.full((n, 3), -1, np.int32)
    g[0, :2] = (1, 2)
    for i in range(1, n - 2):
        g[i, 0] = i + 2                      # odd nodes follow node 1, even nodes follow node 2
    g[1, 1], g[1, 2] = 37, 39                # node 1's branch scores two more nodes than node 2's
    return values.reshape(-1, 1), g


@pytest.mark.parametrize("gap,accepted", [(2e-7, True), (1e-3, False)])
def test_a_different_walk_is_accepted_only_behind_a_near_tie(gap, accepted):
    x, g = chain_with_a_fork(gap)
    x32 = x.astype(np.float32)
    gap32 = float(x32[1, 0]) - float(x32[2, 0])
    assert (gap32 < 1e-6) == accepted
    q = np.ones((1, 1), np.float32)
    k, ef = 1, 1
    o_ids, _, _, nd, ne = oracle.graph_search(x32, g, 0, q, k, ef)
    # the walk a device would take had its arithmetic ordered nodes 1 and 2 the other way round:
    # the oracle itself on a corpus with the two values exchanged
    y32 = x32.copy()
    y32[[1, 2]] = y32[[2, 1]]
    p_ids, _, _, p_nd, p_ne = oracle.graph_search(y32, g, 0, q, k, ef)
    assert (int(p_nd[0]), int(p_ne[0])) != (int(nd[0]), int(ne[0])), "the fork must change the counters"
    args = (x32, g, q, 0, "f32", [0], k, ef, o_ids[0].tolist(), (int(nd[0]), int(ne[0])),
            p_ids[0].tolist(), (int(p_nd[0]), int(p_ne[0])))
    if accepted:
        pairs = explain_divergence(*args)
        assert [(a, b) for a, b, _ in pairs] == [(2, 1)] and pairs[0][2] == pytest.approx(gap32)
    else:
        with pytest.raises(AssertionError, match="no near-tie"):
            explain_divergence(*args)


def test_explaining_walk_is_the_oracles_search():
    n, d, R = 300, 16, 6
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    q = x[:5] + 0.1 * rng.standard_normal((5, d)).astype(np.float32)
    g = rng.integers(-1, n + 2, size=(n, R)).astype(np.int32)
    for ef, entries in ((1, [4]), (8, [4]), (40, [9, 9, 250, -1, 3])):
        ids, _, _, nd, ne = oracle.graph_search(x, g, 0, q, min(3, ef), ef, entries=np.tile(np.array(entries, np.int32), (5, 1)))
        for b in range(5):
            got = walk(lambda v: oracle.score(x, q, b, v), lambda v: g[v], n, entries, min(3, ef), ef)
            assert got[0] == [i for i in ids[b].tolist() if i >= 0]
            assert got[1:3] == (int(nd[b]), int(ne[b]))


def test_topk_rule_rejects_a_clear_miss_and_accepts_a_boundary_tie():
    x = np.array([[0.9], [0.5], [0.5 - 2e-5], [0.1]], np.float32)
    q = np.ones((1, 1), np.float32)
    o_ids, _, o64 = oracle.flat_search(x, q, 2)
    assert o_ids[0].tolist() == [0, 1]
    s = lambda ids: np.array([[float(x[i, 0]) for i in ids]], np.float32)
    assert compare_topk(np.array([[0, 1]]), s([0, 1]), o_ids, o64, x, q) == (1, 0, 1)
    assert compare_topk(np.array([[0, 2]]), s([0, 2]), o_ids, o64, x, q) == (0, 1, 1)     # 2e-5 from rank k
    with pytest.raises(AssertionError):
        compare_topk(np.array([[0, 3]]), s([0, 3]), o_ids, o64, x, q)                      # 0.4 from rank k
    with pytest.raises(AssertionError):
        compare_topk(np.array([[1, 2]]), s([1, 2]), o_ids, o64, x, q)                      # the clear best is lost
