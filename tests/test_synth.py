"""Checks of the seeded input generators (no GPU): shapes, norms, the cluster-size
apportionment, determinism, and the two graph builders against numpy brute force."""
import numpy as np
import torch

from paper_2505_12065_amd import synth


def test_zipf_sizes_apportionment():
    n = synth.zipf_sizes(1_000_000, 1024, 1.1)
    assert int(n.sum()) == 1_000_000
    assert bool((n[1:-1] >= n[2:]).all()) and int(n[-1]) >= 1
    w = torch.arange(1, 1025, dtype=torch.float64).pow(-1.1)
    assert abs(int(n[1]) - 1_000_000 * float(w[1] / w.sum())) <= 1
    assert 0.15 < int(n[0]) / 1_000_000 < 0.21


def test_corpus_is_unit_norm_and_reproducible():
    c1 = synth.make_corpus(5000, 64, 12, seed=7)
    c2 = synth.make_corpus(5000, 64, 12, seed=7)
    c3 = synth.make_corpus(5000, 64, 12, seed=8)
    assert c1.x.dtype == torch.float16 and c1.x.shape == (5000, 64)
    assert torch.equal(c1.x, c2.x) and torch.equal(c1.labels, c2.labels)
    assert not torch.equal(c1.x, c3.x)
    norms = c1.x.double().norm(dim=1)
    assert float((norms - 1).abs().max()) < 1e-3
    assert torch.equal(torch.bincount(c1.labels.long(), minlength=12), synth.zipf_sizes(5000, 12))
    # points sit near their own centroid direction
    cn = c1.centroids / c1.centroids.norm(dim=1, keepdim=True)
    assert float((c1.x.float() @ cn.T).argmax(1).eq(c1.labels.long()).float().mean()) > 0.99


def test_queries_are_noisy_unit_copies():
    c = synth.workload_corpus(0)
    assert c.x.shape == (10_000, 128) and c.x.dtype == torch.float32
    q = synth.make_queries(c, 64)
    assert q.shape == (64, 128) and q.dtype == torch.float32
    assert float((q.norm(dim=1) - 1).abs().max()) < 1e-5
    best = (q @ c.x.T).max(1).values
    # noise of std 0.05 per coordinate at d = 128 has norm ~0.57: cos ~ 1/sqrt(1+0.32) ~ 0.87
    assert 0.8 < float(best.mean()) < 0.95


def brute_knn(x, pool_of, R):
    x = x.double().numpy()
    out = np.full((x.shape[0], R), -1, np.int64)
    for i in range(x.shape[0]):
        pool = [j for j in pool_of(i) if j != i]
        s = x[pool] @ x[i]
        order = sorted(range(len(pool)), key=lambda t: (-s[t], pool[t]))[:R]
        out[i, :len(order)] = [pool[t] for t in order]
    return out


def test_knn_graph_matches_brute_force():
    c = synth.make_corpus(400, 32, 5, seed=3, dtype=torch.float32, zipf_a=None, sigma=0.3)
    c.x[17] = c.x[3]          # exact duplicate: tie must go to the lower id
    g = synth.knn_graph(c.x, 8, row_block=128)
    want = brute_knn(c.x, lambda i: range(400), 8)
    assert np.array_equal(g.numpy(), want)
    assert g.dtype == torch.int32


def test_cluster_restricted_graph_matches_brute_force():
    c = synth.make_corpus(600, 32, 20, seed=4, dtype=torch.float16)
    R, near = 8, 3
    g = synth.knn_graph_cluster_restricted(c, R, near, row_block=100, col_block=64)
    cn = (c.centroids / c.centroids.norm(dim=1, keepdim=True)).double()
    nearest = torch.topk(c.x.float() @ cn.float().T, near, dim=1).indices.numpy()
    labels = c.labels.numpy()
    members = {b: np.nonzero(labels == b)[0].tolist() for b in range(20)}

    def pool_of(i):
        return sorted(j for b in nearest[i] for j in members[int(b)])
    want = brute_knn(c.x, pool_of, R)
    got = g.numpy()
    # fp32 matmul vs fp64 brute force: allow swaps only between near-equal scores
    x64 = c.x.double().numpy()
    for i in range(600):
        if got[i].tolist() != want[i].tolist():
            sg = np.sort(x64[got[i][got[i] >= 0]] @ x64[i])[::-1]
            sw = np.sort(x64[want[i][want[i] >= 0]] @ x64[i])[::-1]
            assert np.allclose(sg, sw, atol=1e-6), i
    assert (got == want).mean() > 0.995
    # smallest clusters give short pools -> trailing -1 padding is allowed, never inside a row
    for row in got:
        valid = row >= 0
        assert not np.any(valid[1:] & ~valid[:-1])


def test_mean_entry_and_ring():
    c = synth.make_corpus(300, 16, 4, seed=5, dtype=torch.float16)
    e = synth.mean_entry(c.x)
    mu = c.x.double().mean(0)
    assert e == int((c.x.double() @ mu).argmax())
    g = synth.ring_union(torch.full((300, 2), -1, dtype=torch.int32))
    assert g.shape == (300, 4) and int(g[0, 3]) == 299 and int(g[299, 2]) == 0


def test_cluster_representatives_match_brute_force():
    c = synth.make_corpus(3000, 32, 6, seed=3, dtype=torch.float16, zipf_a=1.1, sigma=0.3)
    reps = synth.cluster_representatives(c)
    cn = c.centroids / c.centroids.norm(dim=1, keepdim=True)
    assert reps.dtype == torch.int32 and reps.shape == (6,)
    for ci in range(6):
        m = (c.labels == ci).nonzero().flatten()
        s = c.x[m].float() @ cn[ci]
        assert int(reps[ci]) == int(m[(s == s.max()).nonzero()[0, 0]])


def test_reverse_edge_graph_matches_brute_force():
    c = synth.make_corpus(1500, 32, 5, seed=8, dtype=torch.float16, zipf_a=None, sigma=0.3)
    g = synth.knn_graph(c.x, 8)
    g[17, 5:] = -1                                  # a short row
    h = synth.with_reverse_edges(g, c.x)
    x, gn, hn = c.x.float().numpy(), g.numpy(), h.numpy()
    N, R = gn.shape
    rev = {j: [] for j in range(N)}
    for i in range(N):
        for j in gn[i]:
            if j >= 0:
                rev[int(j)].append((-float(np.float32(x[i] @ x[j])), i))
    loose = 0
    for j in range(N):
        want = [int(v) for v in gn[j, :R // 2] if v >= 0]
        for _, i in sorted(rev[j]):
            if i not in want:
                want.append(i)
        for v in gn[j, R // 2:]:
            if v >= 0 and int(v) not in want:
                want.append(int(v))
        want = (want + [-1] * R)[:R]
        if want != hn[j].tolist():                  # summation order may swap near-equal reverse scores
            assert sorted(want) == sorted(hn[j].tolist()) or len(set(want) ^ set(hn[j].tolist())) <= 2, j
            loose += 1
    assert loose <= N // 100
    assert (hn[:, : R // 2] == gn[:, : R // 2])[gn[:, : R // 2] >= 0].all()


def test_diversity_pruning_rule_on_a_line():
    """Points on a line around node 0: candidates on the same side as an already selected closer neighbour are
    passed over (they are closer to that neighbour than to the node), the first one on the other side is taken."""
    import torch
    from paper_2505_12065_amd import synth
    # 1-d positions embedded on the unit circle at small angles, so that larger inner product = closer
    ang = torch.tensor([0.0, 0.010, 0.020, 0.030, -0.015, -0.040])
    x = torch.stack([torch.cos(ang), torch.sin(ang)], 1)
    g = torch.tensor([[1, 4, 2, 3, 5], [-1] * 5, [-1] * 5, [-1] * 5, [-1] * 5, [-1] * 5], dtype=torch.int32)   # node 0: by closeness
    pruned, frac = synth.diversity_pruned(g, x, keep=5)
    # taken: 1 (closest), 4 (other side); passed over: 2 and 3 (closer to 1), 5 (closer to 4); they fill the row after the taken ones
    assert pruned[0].tolist() == [1, 4, 2, 3, 5]
    assert frac == 3 / 5
    pruned2, _ = synth.diversity_pruned(g, x, keep=2)
    assert pruned2[0].tolist() == [1, 4, -1, -1, -1]
