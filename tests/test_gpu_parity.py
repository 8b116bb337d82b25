"""GPU parity: the HIP library, called through its C ABI (via the ctypes binding),
against the CPU oracle on the same seeded inputs.  Integer outputs (ids) must be
identical up to the stated near-tie rule, scores within 1e-4 absolute."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_12065_amd as ann
from paper_2505_12065_amd import synth
from parity import TOL, compare_topk, explain_divergence, np_dtype_name, recall, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def flat_both(x, q, k):
    """x, q: cpu tensors.  Returns gpu (ids, scores) as numpy and oracle (ids, sc, sc64)."""
    ids, sc = ann.ann_flat_search_typed(x.to(DEV), q.to(DEV), k)
    torch.cuda.synchronize()
    name = np_dtype_name(x)
    o = oracle.flat_search(to_np(x), to_np(q), k, dtype=name)
    return ids.cpu().numpy(), sc.cpu().numpy(), o


# ------------------------------------------------------------------ configuration 0 (tiny, fp32)

@pytest.fixture(scope="module")
def cfg0():
    c = synth.workload_corpus(0)
    q = synth.make_queries(c, 64)
    g = synth.knn_graph(c.x, 16)
    return c, q, g


def test_cfg0_flat_fp32(cfg0):
    c, q, _ = cfg0
    say("cfg0 flat: N=10000 d=128 fp32 B=64 k=10")
    ids, sc, (o_ids, o_sc, o_sc64) = flat_both(c.x, q, 10)
    strict, tolerant, n = compare_topk(ids, sc, o_ids, o_sc64, c.x.numpy(), q.numpy())
    say(f"cfg0 flat strict={strict}/{n} tolerant={tolerant}")
    assert strict >= n - 2


def test_cfg0_graph_fp32(cfg0):
    c, q, g = cfg0
    say("cfg0 graph: 16-NN graph, entry 0, ef=32, k=10")
    ids, sc = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 0, q.to(DEV), 10, 32)
    torch.cuda.synchronize()
    o_ids, o_sc, o_sc64, nd, ne = oracle.graph_search(c.x.numpy(), g.numpy(), 0, q.numpy(), 10, 32)
    strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, c.x.numpy(), q.numpy())
    f_ids, _, _ = oracle.flat_search(c.x.numpy(), q.numpy(), 10)
    say(f"cfg0 graph strict={strict}/{n} recall@10 gpu={recall(ids.cpu().numpy(), f_ids):.3f} "
        f"oracle={recall(o_ids, f_ids):.3f} n_dist={nd.mean():.0f} n_expand={ne.mean():.0f}")
    assert strict >= n - 2


# ------------------------------------------------------------------ flat: shapes, tails, dtypes

@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N,d,B,k", [
    (16 * 37 + 5, 768, 1, 3),       # ragged last tile
    (1, 64, 2, 1),                  # single row
    (7, 32, 3, 7),                  # k = N, fewer rows than a tile
    (5000, 136, 17, 10),            # d not a multiple of 32, B not a multiple of 16
    (20000, 768, 64, 3),            # four query groups in one pass
    (9001, 256, 70, 16),            # two passes, k = K_MAX
    (4099, 384, 130, 5),            # the paper's embedding width
    (3000, 1024, 33, 4),
    (5000, 768, 100, 3),            # matrix-core path, 128-query tile, ragged corpus tile
    (777, 64, 300, 4),              # matrix-core path, two 256-query tiles, second one ragged
    (70001, 256, 129, 1),           # matrix-core path, many tiles per slab
    (100, 32, 2100, 2),             # more query tiles than tile groups; corpus smaller than a tile
    (50_000, 768, 32, 3),           # two query groups, many tiles per wave
    (2049, 96, 20, 10),             # ... ragged tile, k > 4
    (300, 4096, 9, 2),              # largest d
    (600_001, 64, 200, 3),          # matrix-core path with the sampling pass, one query tile
    (300_000, 32, 600, 4),          # ... three query tiles
    (131_072 + 77, 128, 96, 5),     # matrix-core path with candidate arrays (k > 4), 128-query tile
    (200_003, 64, 300, 16),         # ... two 256-query tiles, k = K_MAX
    (150_000, 96, 130, 10),         # ... ragged sample tile
    (131_072, 64, 1, 5),            # streaming path with candidate arrays (k > 4), one query
    (140_000, 136, 17, 10),         # ... d not a multiple of 32
    (150_001, 72, 70, 7),           # ... two passes of queries
])
def test_flat_shapes(dtype, N, d, B, k):
    say(f"flat shapes: dtype={dtype} N={N} d={d} B={B} k={k}")
    c = synth.make_corpus(N, d, min(8, N), seed=N + d, dtype=dtype, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, B)
    ids, sc, (o_ids, o_sc, o_sc64) = flat_both(c.x, q, k)
    strict, tolerant, n = compare_topk(ids, sc, o_ids, o_sc64, to_np(c.x), to_np(q), dtype=np_dtype_name(c.x))
    assert strict >= n - max(2, n // 20), (strict, n)


@pytest.mark.parametrize("dtype,N,d,B,k", [
    (torch.float16, 30_000, 128, 9, 16),        # streaming kernel, lists of 16
    (torch.float16, 200_000, 64, 20, 16),       # streaming kernel, candidate arrays
    (torch.bfloat16, 70_000, 96, 300, 4),       # matrix-core kernel, lists, sampled thresholds
    (torch.float16, 700_000, 64, 100, 3),       # matrix-core kernel, the sample is the first tile of every slab
    (torch.float16, 150_000, 128, 260, 16),     # matrix-core kernel, candidate arrays
    (torch.float32, 9_000, 64, 11, 16),         # fp32 kernel
    (torch.float16, 40, 64, 5, 16),             # pages run past the end of a small corpus
    (torch.float16, 40, 64, 200, 16),           # the same through the matrix-core kernel: the sample has < k rows
    (torch.bfloat16, 300, 96, 700, 16),         # ragged last tile of 256 rows, threshold of -inf, three query tiles
    (torch.float16, 5000, 64, 90, 9),           # candidate arrays on a corpus of a few thousand rows
])
def test_flat_continuation_pages(dtype, N, d, B, k):
    """The next k rows after a boundary pair, three pages in a row: each side continues from its own last
    pair (the GPU from its fp32 score, the oracle from its binary64 score), page against page, and the GPU's
    pages together against one oracle answer of 3 k rows.  A quarter of the corpus is a copy of other
    rows, so page boundaries cut through tied scores."""
    say(f"flat continuation: dtype={dtype} N={N} d={d} B={B} k={k}")
    c = synth.make_corpus(N, d, 8, seed=N % 89, dtype=dtype, zipf_a=None, sigma=0.3)
    x = c.x.clone()
    x[N // 2: N // 2 + N // 4] = x[: N // 4]
    q = synth.make_queries(c, B)
    xd, qd = x.to(DEV), q.to(DEV)
    name = np_dtype_name(x)
    xn, qn = to_np(x), to_np(q)
    after_gpu, after_o, pages = None, None, []
    for page in range(3):
        ids, sc = ann.ann_flat_search_typed(xd, qd, k, after=after_gpu)
        torch.cuda.synchronize()
        o_ids, o_sc, o_sc64 = oracle.flat_search(xn, qn, k, after=after_o, dtype=name)
        assert int(ids.max()) < N and int(ids.min()) >= -1, page     # padding is -1, never a row number >= N
        strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, xn, qn, dtype=name)
        assert strict >= n - max(1, n // 50), (page, strict, n)
        pages.append(ids.cpu().numpy())
        if (o_ids[:, -1] < 0).any():
            break
        after_gpu = (sc[:, -1].contiguous(), ids[:, -1].contiguous())
        after_o = (o_sc64[:, -1], o_ids[:, -1])
    got = np.concatenate(pages, 1)
    want, _, _ = oracle.flat_search(xn, qn, min(N, got.shape[1]), dtype=name)
    exact_rows = sum(got[b, :want.shape[1]].tolist() == want[b].tolist() for b in range(B))
    say(f"  pages concatenated equal one answer of {want.shape[1]} rows for {exact_rows}/{B} queries")
    assert exact_rows >= B - max(1, B // 50)
    for b in range(B):
        row = [i for i in got[b].tolist() if i >= 0]
        assert len(set(row)) == len(row), b                     # no row twice
    if N == 40:
        assert (got[:, 40:] == -1).all() and (np.sort(got[:, :40], 1) == np.arange(40)).all()


def test_flat_ties_go_to_lower_id():
    c = synth.make_corpus(4000, 128, 4, seed=5, dtype=torch.float16, zipf_a=None, sigma=0.3)
    x = c.x.clone()
    for dst in (77, 1999, 3998, 16, 17):
        x[dst] = x[1000]
    q = x[1000:1001].clone()
    ids, sc = ann.ann_flat_search_typed(x.to(DEV), q.to(DEV), 8)
    torch.cuda.synchronize()
    assert ids[0, :6].tolist() == [16, 17, 77, 1000, 1999, 3998]
    assert float(sc[0, 0]) == float(sc[0, 5])
    o_ids, _, _ = oracle.flat_search(x.numpy(), q.numpy(), 8)
    assert ids.cpu().numpy().tolist() == o_ids.tolist()


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("B,a,b,n_wide,n_stream", [(80, 7, 66, 1, 0), (20, 7, 13, 0, 1)])
def test_flat_candidate_array_overflow_is_repaired(dtype, B, a, b, n_wide, n_stream):
    """k > 4 on a large corpus collects, per query, the rows that reach a sampled bound of the
    k-th best score (large batches on the matrix cores, small ones in the streaming kernel).  Thousands of rows tied at the top overflow that array; such a query is then
    recomputed by the streaming kernel while the others keep their results.  Rows sorted by
    cluster (the sample must still represent every cluster) are covered as well."""
    N, d, k = 140_000, 64, 6
    c = synth.make_corpus(N, d, 16, seed=31, dtype=dtype, zipf_a=None, sigma=0.3)
    order = torch.argsort(c.labels.cpu(), stable=True)
    x = c.x.cpu()[order].contiguous()
    gen = torch.Generator().manual_seed(3)
    copies = torch.randperm(N, generator=gen)[:6000]
    x[copies] = x[int(copies[0])].clone()
    q = synth.make_queries(c, B).cpu()
    q[a] = x[int(copies[0])]
    q[b] = x[int(copies[0])]
    say(f"flat candidate arrays with 6000 tied rows: dtype={dtype} B={B}")
    ann.ann_timing_enable(True)
    ids, sc, (o_ids, o_sc, o_sc64) = flat_both(x, q, k)
    wide, stream = ann.ann_timing_read(ann.binding.KERNEL_FLAT_WIDE), ann.ann_timing_read(ann.binding.KERNEL_FLAT_STREAM)
    ann.ann_timing_enable(False)
    assert wide[0] == n_wide and stream[0] == n_stream          # the main pass; the repair pass is not recorded
    low = sorted(copies.tolist())[:k]
    assert ids[a].tolist() == low and ids[b].tolist() == low and o_ids[a].tolist() == low
    strict, tolerant, n = compare_topk(ids, sc, o_ids, o_sc64, to_np(x), to_np(q), dtype=np_dtype_name(x))
    assert strict >= n - 2, (strict, n)


def test_flat_short_entry_point_and_reuse_of_outputs():
    c = synth.make_corpus(3000, 64, 4, seed=9, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 5)
    xd, qd = c.x.to(DEV), q.to(DEV)
    ids = torch.full((5, 3), -7, dtype=torch.int32, device=DEV)
    sc = torch.zeros(5, 3, device=DEV)
    r_ids, r_sc = ann.ann_flat_search(xd, qd, 3, ids=ids, scores=sc)
    assert r_ids is ids and r_sc is sc
    t_ids, t_sc = ann.ann_flat_search_typed(xd, qd, 3)
    torch.cuda.synchronize()
    assert torch.equal(ids, t_ids) and torch.equal(sc, t_sc)
    # a side stream works too
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        s_ids, s_sc = ann.ann_flat_search_typed(xd, qd, 3)
    s.synchronize()
    assert torch.equal(s_ids, t_ids)


def test_caller_owned_workspace():
    """ann_set_workspace: the searches run in the caller's buffer, give the same results, and a
    buffer that is too small is an error, not an allocation."""
    c = synth.make_corpus(40_000, 256, 8, seed=3, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 96)
    g = synth.ring_union(synth.knn_graph(c.x.to(DEV), 10).cpu()).contiguous()
    xd, qd, gd = c.x.to(DEV), q.to(DEV), g.to(DEV)
    want = ann.ann_flat_search_typed(xd, qd, 3)
    want_g = ann.ann_graph_search_nonstall_typed(xd, gd, 1, qd, 3, 40, tau=0.8, window=50)
    torch.cuda.synchronize()
    need = max(ann.ann_flat_workspace_bytes(40_000, 256, torch.float16, 96, 3), ann.ann_graph_nonstall_workspace_bytes(40_000, 96))
    buf = torch.full((need + 4096,), 0xAB, dtype=torch.uint8, device=DEV)
    try:
        ann.ann_set_workspace(buf)
        got = ann.ann_flat_search_typed(xd, qd, 3)
        got_g = ann.ann_graph_search_nonstall_typed(xd, gd, 1, qd, 3, 40, tau=0.8, window=50)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
        for a, b in zip(got_g, want_g):
            assert torch.equal(a, b)
        assert bool((buf[:1024] != 0xAB).any())                  # the buffer was really used
        ann.ann_set_workspace(buf[:256])
        with pytest.raises(ann.AnnError) as e:
            ann.ann_flat_search_typed(xd, qd, 3)
        assert e.value.code == ann.binding.ANN_ERR_NOMEM
    finally:
        ann.ann_set_workspace(None)
    again = ann.ann_flat_search_typed(xd, qd, 3)
    torch.cuda.synchronize()
    assert torch.equal(again[0], want[0])


def test_flat_is_deterministic():
    c = synth.make_corpus(50_000, 768, 32, seed=21, dtype=torch.float16)
    q = synth.make_queries(c, 48)
    xd, qd = c.x.to(DEV), q.to(DEV)
    a = ann.ann_flat_search_typed(xd, qd, 3)
    b = ann.ann_flat_search_typed(xd, qd, 3)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_error_codes_on_device():
    x = torch.zeros(100, 64, dtype=torch.float16, device=DEV)
    q = torch.zeros(2, 64, dtype=torch.float16, device=DEV)
    g = torch.zeros(100, 4, dtype=torch.int32, device=DEV)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_flat_search_typed(x, q, 101)
    assert e.value.code == -1
    with pytest.raises(ann.AnnError) as e:
        ann.ann_graph_search_typed(x, g, 0, q, 5, 4)
    assert e.value.code == -1
    with pytest.raises(ann.AnnError) as e:
        ann.ann_graph_search(x, g, 0, q, 1, 4)
    assert e.value.code == -3
    ann.ann_register_corpus(x)
    ann.ann_graph_search(x, g, 0, q, 1, 4)
    torch.cuda.synchronize()
    ann.ann_unregister_corpus(x)


def test_empty_batches_are_no_ops():
    """B = 0 (and n = 0 for the helpers) returns at once with success, launches nothing and
    touches nothing, whatever the other arguments are."""
    x = torch.zeros(100, 64, dtype=torch.float16, device=DEV)
    g = torch.zeros(100, 4, dtype=torch.int32, device=DEV)
    q0 = torch.zeros(0, 64, dtype=torch.float16, device=DEV)
    ann.ann_timing_enable(True)
    ids, sc = ann.ann_flat_search_typed(x, q0, 3)
    assert ids.shape == (0, 3) and sc.shape == (0, 3)
    ids, sc = ann.ann_graph_search_typed(x, g, 0, q0, 3, 8)
    assert ids.shape == (0, 3)
    e0 = torch.zeros(0, dtype=torch.int32, device=DEV)
    ids, sc = ann.ann_graph_search_entries_typed(x, g, e0, q0, 3, 8)
    assert ids.shape == (0, 3)
    out = ann.ann_graph_search_nonstall_typed(x, g, 0, q0, 3, 8)
    assert out[0].shape == (0, 3) and out[2].shape == (0, 3) and out[3].shape == (0,)
    assert ann.ann_gather_ids(torch.arange(5, dtype=torch.int32, device=DEV), e0).shape == (0,)
    torch.cuda.synchronize()
    for code in (ann.binding.KERNEL_FLAT_STREAM, ann.binding.KERNEL_FLAT_WIDE, ann.binding.KERNEL_GRAPH):
        assert ann.ann_timing_read(code)[0] == 0
    ann.ann_timing_enable(False)
    lib = ann.binding.lib()
    assert lib.ann_flat_search_typed(None, 0, 0, 0, None, 0, 0, None, None, None) == 0      # nothing is looked at


# ------------------------------------------------------------------ configuration 1 (flat, fp16, d = 768)

@pytest.fixture(scope="module")
def cfg1_scaled():
    """Configuration 1 at a tenth of its size: the oracle can do every query."""
    c = synth.workload_corpus(1, scale=0.1)
    q = synth.make_queries(c, 512)
    return c, q


@pytest.mark.parametrize("B", [1, 16, 64, 256, 512])
def test_cfg1_scaled_flat_all_batches(cfg1_scaled, B):
    c, q = cfg1_scaled
    q = q[:B].contiguous()
    say(f"cfg1/10 flat: N={c.x.shape[0]} d=768 fp16 B={B} k=3")
    ids, sc, (o_ids, o_sc, o_sc64) = flat_both(c.x, q, 3)
    strict, tolerant, n = compare_topk(ids, sc, o_ids, o_sc64, c.x.numpy(), q.numpy())
    say(f"cfg1/10 B={B}: strict={strict}/{n} tolerant={tolerant}")
    assert strict >= n - max(1, n // 50)


# ------------------------------------------------------------------ graph: shapes and special cases

@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
def test_graph_ef_at_least_n_on_connected_graph_is_exact(dtype):
    c = synth.make_corpus(600, 64, 6, seed=31, dtype=dtype, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 9)
    g = synth.ring_union(synth.knn_graph(c.x, 6))
    ids, sc = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 17, q.to(DEV), 10, 600)
    torch.cuda.synchronize()
    f_ids, _, f64 = oracle.flat_search(to_np(c.x), to_np(q), 10, dtype=np_dtype_name(c.x))
    compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), f_ids, f64, to_np(c.x), to_np(q), dtype=np_dtype_name(c.x))


@pytest.mark.parametrize("R,ef,k", [(1, 1, 1), (3, 2, 2), (32, 8, 3), (33, 64, 10), (70, 40, 7), (16, 300, 16)])
def test_graph_shapes(R, ef, k):
    say(f"graph shapes: R={R} ef={ef} k={k}")
    N, d = 5000, 136
    c = synth.make_corpus(N, d, 10, seed=R * 100 + ef, dtype=torch.float16, zipf_a=None, sigma=0.4)
    q = synth.make_queries(c, 21)
    gen = torch.Generator().manual_seed(R)
    g = synth.knn_graph(c.x, max(1, R // 2))
    rnd = torch.randint(-1, N + 3, (N, R - g.shape[1]), generator=gen, dtype=torch.int32)   # junk ids, some invalid
    g = torch.cat([g, rnd], 1).contiguous()
    g[5, : min(R, 2)] = 5                                                                    # self loops
    ids, sc = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 3, q.to(DEV), k, ef)
    torch.cuda.synchronize()
    o_ids, o_sc, o_sc64, nd, ne = oracle.graph_search(c.x.numpy(), g.numpy(), 3, q.numpy(), k, ef)
    strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, c.x.numpy(), q.numpy())
    assert strict >= n - 2, (strict, n)


@pytest.mark.parametrize("ef,R,dtype", [(2049, 32, torch.float16), (3000, 12, torch.float16), (6000, 32, torch.bfloat16),
                                        (16384, 40, torch.float16), (5000, 32, torch.float32), (16384, 32, torch.float16),
                                        (8192, 24, torch.float16)])
def test_graph_long_lists(ef, R, dtype):
    """Lists longer than 2048 entries, exact visited bitset: the two-level list (R <= 32) and the single
    buffer merged in place (R > 32); results and counters against the oracle."""
    N = 30_000
    say(f"graph long list: ef={ef} R={R} {dtype}")
    c = synth.make_corpus(N, 64, 12, seed=ef, dtype=dtype, zipf_a=None, sigma=0.35)
    q = synth.make_queries(c, 6)
    g = synth.ring_union(synth.knn_graph(c.x.to(DEV), R - 2).cpu()).contiguous()
    ids, sc = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 7, q.to(DEV), 5, ef)
    torch.cuda.synchronize()
    name = np_dtype_name(c.x)
    o_ids, _, o_sc64, nd, ne = oracle.graph_search(to_np(c.x), g.numpy(), 7, to_np(q), 5, ef, dtype=name)
    strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, to_np(c.x), to_np(q), dtype=name)
    say(f"  strict {strict}/{n}, oracle expansions {ne.mean():.0f}, scored {nd.mean():.0f}")
    assert strict >= n - 1
    # the counters of the long-list path through the non-stall entry point are the oracle's
    ids_ns, _, stats, _ = ann.ann_graph_search_nonstall_typed(c.x.to(DEV), g.to(DEV), 7, q.to(DEV), 5, ef, tau=float("inf"))
    ids_ns = ids_ns.cpu().numpy()
    st = stats.cpu().numpy()
    for b in range(q.shape[0]):
        if (int(st[b, 1]), int(st[b, 2])) == (int(nd[b]), int(ne[b])):
            continue
        # another walk than the oracle's: only the reversal of a near-tie (fp64 gap below 1e-6) may cause it
        pairs = explain_divergence(to_np(c.x), g.numpy(), to_np(q), b, name, [7], 5, ef, o_ids[b].tolist(),
                                   (int(nd[b]), int(ne[b])), ids_ns[b].tolist(), (int(st[b, 1]), int(st[b, 2])))
        say(f"  query {b}: walk differs at a near-tie: " + ", ".join(f"nodes {a}/{c2} gap {gap:.2e}" for a, c2, gap in pairs))


@pytest.mark.parametrize("ef,R,k", [(16, 8, 5), (200, 32, 10), (700, 32, 16), (48, 40, 7), (2100, 32, 16), (2600, 16, 8)])
def test_graph_ties_go_to_lower_id(ef, R, k):
    """Every vector occurs four times under scattered ids, so a query scores the copies exactly alike (in fp32
    on the GPU as in fp64 in the oracle) and the order (score descending, id ascending) decides every one of
    those ties: in the list positions, among the neighbours of one expansion, in the choice of the next node,
    at the k-th place.  Ids must match the oracle's exactly."""
    say(f"graph with tied scores: ef={ef} R={R} k={k}")
    N, d = 4000, 64
    base = synth.make_corpus(N // 4, d, 8, seed=ef + R, dtype=torch.float16, zipf_a=None, sigma=0.4)
    gen = torch.Generator().manual_seed(ef)
    where = torch.randperm(N, generator=gen)                      # copy j of vector i sits at row where[4 i + j]
    x = torch.empty(N, d, dtype=torch.float16)
    x[where] = base.x.repeat_interleave(4, 0)
    q = synth.make_queries(base, 24)
    g = synth.ring_union(synth.knn_graph(x, R - 2)).contiguous()
    ids, sc = ann.ann_graph_search_typed(x.to(DEV), g.to(DEV), 5, q.to(DEV), k, ef)
    torch.cuda.synchronize()
    o_ids, o_sc, o_sc64, nd, ne = oracle.graph_search(x.numpy(), g.numpy(), 5, q.numpy(), k, ef)
    assert (o_sc[:, 0] == o_sc[:, 1]).any(), "the workload is meant to have ties at the top"
    assert np.array_equal(ids.cpu().numpy(), o_ids)
    assert np.abs(sc.cpu().numpy() - o_sc64).max() < 1e-4
    # the same through the maturity-exit entry point with the exit switched off, counters included
    n_ids, n_sc, stats, _ = ann.ann_graph_search_nonstall_typed(x.to(DEV), g.to(DEV), 5, q.to(DEV), k, ef, tau=float("inf"))
    torch.cuda.synchronize()
    assert np.array_equal(n_ids.cpu().numpy(), o_ids)
    st = stats.cpu().numpy()
    assert np.array_equal(st[:, 1], nd) and np.array_equal(st[:, 2], ne)


@pytest.mark.parametrize("seed,cases,n_max,r_choices,ef_choices", [
    (2024, 30, 4000, [1, 2, 5, 8, 16, 31, 32, 33, 48], [1, 3, 17, 64, 65, 200, 256, 257, 400, 512, 513, 900]),
    # the two-level list (search ranges beyond 512, at most 32 slots per node): lists that never fill, lists
    # that hold most of the graph, rebuilds every few expansions (R = 32) and every few hundred (R = 1, 2)
    (77, 16, 7000, [1, 2, 5, 16, 32], [513, 600, 770, 1500, 2049, 2500, 5000]),
])
def test_graph_random_configurations(seed, cases, n_max, r_choices, ef_choices):
    """Seeded draws of (N, d, R, ef, k, dtype, B) with junk ids, repeated ids and repeated vectors in
    the inputs: every list length regime (up to 64, up to 256, up to 512, beyond), both loops (R <= 32 and
    R > 32) and both entry points against the oracle, counters of the maturity variant included."""
    rng = np.random.default_rng(seed)
    total = strict_total = 0
    for case in range(cases):
        N = int(rng.integers(40, n_max))
        d = int(rng.choice([8, 16, 24, 64, 72, 136, 256, 520]))
        R = int(rng.choice(r_choices))
        ef = int(rng.choice(ef_choices))
        k = int(rng.integers(1, min(ef, 20) + 1))
        B = int(rng.integers(1, 12))
        dtype = [torch.float16, torch.bfloat16, torch.float32][int(rng.integers(0, 3))]
        say(f"graph random case {case}: N={N} d={d} R={R} ef={ef} k={k} B={B} {dtype}")
        c = synth.make_corpus(N, d, max(2, N // 300), seed=1000 + case, dtype=dtype, zipf_a=None, sigma=0.4)
        x = c.x.clone()
        gen = torch.Generator().manual_seed(case)
        copies = torch.randint(0, N, (N // 10,), generator=gen)
        x[copies] = x[torch.randint(0, N, (N // 10,), generator=gen)].clone()        # repeated vectors: tied scores
        q = synth.make_queries(c, B)
        nn_ = max(1, min(R, N - 1) // 2)
        g = synth.knn_graph(x, nn_)
        junk = torch.randint(-1, N + 2, (N, R - g.shape[1]), generator=gen, dtype=torch.int32)
        g = torch.cat([g, junk], 1)[:, :R].contiguous()
        g[:, -1] = (torch.arange(N, dtype=torch.int32) + 1) % N                       # a ring keeps it connected
        if R >= 2:
            g[::7, 0] = g[::7, R - 1]                                                 # an id named twice in a row
        entry = int(rng.integers(0, N))
        name = np_dtype_name(x)
        xn, qn, gn = to_np(x), to_np(q), g.numpy()
        ids, sc = ann.ann_graph_search_typed(x.to(DEV), g.to(DEV), entry, q.to(DEV), k, ef)
        n_ids, n_sc, stats, _ = ann.ann_graph_search_nonstall_typed(x.to(DEV), g.to(DEV), entry, q.to(DEV), k, ef,
                                                                    tau=float("inf"))
        torch.cuda.synchronize()
        o_ids, _, o_sc64, nd, ne = oracle.graph_search(xn, gn, entry, qn, k, ef, dtype=name)
        st, _, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, xn, qn, dtype=name)
        compare_topk(n_ids.cpu().numpy(), n_sc.cpu().numpy(), o_ids, o_sc64, xn, qn, dtype=name)
        assert np.array_equal(ids.cpu().numpy(), n_ids.cpu().numpy()), "the two entry points disagree"
        same = np.all(ids.cpu().numpy() == o_ids, axis=1)
        stn = stats.cpu().numpy()
        assert np.array_equal(stn[same, 1], nd[same]) and np.array_equal(stn[same, 2], ne[same]), (stn, nd, ne)
        total += n
        strict_total += st
    say(f"  {strict_total}/{total} queries with ids identical to the oracle's")
    assert strict_total >= total - max(2, total // 50)


@pytest.mark.parametrize("N,d,B,dtype", [(20_000, 64, 3000, torch.float16), (6000, 776, 1500, torch.float16),
                                          (5000, 1032, 1400, torch.bfloat16), (5000, 260, 1400, torch.float32)])
def test_graph_batch_larger_than_one_resident_round(N, d, B, dtype):
    """More queries than workgroups fit on the chip at once: later workgroups start in LDS that earlier
    ones left behind, and batches this large run the kernel variant that keeps the query in LDS (three
    workgroups per compute unit; rows longer than 64 chunks go through its second loop).  Every row
    against the oracle."""
    c = synth.make_corpus(N, d, 16, seed=31, dtype=dtype, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, B)
    g = synth.ring_union(synth.knn_graph(c.x.to(DEV), 14).cpu()).contiguous()
    gen = torch.Generator().manual_seed(1)
    entries = torch.randint(0, N, (B, 3), generator=gen, dtype=torch.int32)
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    name = np_dtype_name(c.x)
    xn, qn, gn = to_np(c.x), to_np(q), g.numpy()
    for ef, ent in ((32, None), (32, entries), (600, None)):
        if ent is None:
            ids, sc = ann.ann_graph_search_typed(xd, gd, 9, qd, 3, ef)
        else:
            ids, sc = ann.ann_graph_search_multi_typed(xd, gd, ent.to(DEV), qd, 3, ef)
        torch.cuda.synchronize()
        o_ids, _, o_sc64, _, _ = oracle.graph_search(xn, gn, 9, qn, 3, ef, entries=None if ent is None else ent.numpy(), dtype=name)
        strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, xn, qn, dtype=name)
        say(f"graph N={N} d={d} B={B} ef={ef} entries={'shared' if ent is None else '3 per query'}: strict {strict}/{n}")
        assert strict >= n - max(2, n // 200)
        # a small batch of the same queries runs the other kernel variant: same answers
        few, few_sc = (ann.ann_graph_search_typed(xd, gd, 9, qd[:64].contiguous(), 3, ef) if ent is None else
                       ann.ann_graph_search_multi_typed(xd, gd, ent[:64].contiguous().to(DEV), qd[:64].contiguous(), 3, ef))
        torch.cuda.synchronize()
        assert torch.equal(few, ids[:64])
        assert float((few_sc - sc[:64]).abs().max()) < 1e-5


def test_graph_padding_when_few_nodes_are_reachable():
    c = synth.make_corpus(200, 64, 4, seed=2, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 4)
    g = torch.full((200, 4), -1, dtype=torch.int32)
    g[9, 0] = 11                      # 9 -> 11, nothing else
    ids, sc = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 9, q.to(DEV), 5, 16)
    torch.cuda.synchronize()
    o_ids, o_sc, _, _, _ = oracle.graph_search(c.x.numpy(), g.numpy(), 9, q.numpy(), 5, 16)
    assert ids.cpu().numpy().tolist() == o_ids.tolist()
    assert sorted(ids[0, :2].tolist()) == [9, 11] and ids[0, 2:].tolist() == [-1, -1, -1]
    assert torch.isneginf(sc[:, 2:]).all()


def test_graph_is_deterministic():
    c = synth.make_corpus(20_000, 768, 16, seed=41, dtype=torch.float16)
    q = synth.make_queries(c, 32)
    g = synth.knn_graph(c.x.to(DEV), 32).contiguous()
    xd, qd = c.x.to(DEV), q.to(DEV)
    a = ann.ann_graph_search_typed(xd, g, 0, qd, 3, 64)
    b = ann.ann_graph_search_typed(xd, g, 0, qd, 3, 64)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
def test_graph_per_query_entries(dtype):
    """One entry node per query: each row equals the oracle started from that query's entry; an
    entry that is not a node id yields padding."""
    N = 8000
    c = synth.make_corpus(N, 128, 12, seed=61, dtype=dtype, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 40)
    g = synth.knn_graph(c.x, 12)
    gen = torch.Generator().manual_seed(9)
    entries = torch.randint(0, N, (40,), generator=gen, dtype=torch.int32)
    entries[7], entries[21] = -1, N
    ids, sc = ann.ann_graph_search_entries_typed(c.x.to(DEV), g.to(DEV), entries.to(DEV), q.to(DEV), 5, 40)
    torch.cuda.synchronize()
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    xn, qn, gn = to_np(c.x), to_np(q), g.numpy()
    strict = 0
    for b in range(40):
        e = int(entries[b])
        if e < 0 or e >= N:
            assert ids[b].tolist() == [-1] * 5 and np.isneginf(sc[b]).all()
            continue
        o_ids, _, o_sc64, _, _ = oracle.graph_search(xn, gn, e, qn[b:b + 1], 5, 40)
        st, _, _ = compare_topk(ids[b:b + 1], sc[b:b + 1], o_ids, o_sc64, xn, qn, rows=[b])
        strict += st
    assert strict >= 37
    # the same entry for everyone is the scalar-entry call
    same = torch.full((40,), 11, dtype=torch.int32, device=DEV)
    a = ann.ann_graph_search_entries_typed(c.x.to(DEV), g.to(DEV), same, q.to(DEV), 5, 40)
    b_ = ann.ann_graph_search_typed(c.x.to(DEV), g.to(DEV), 11, q.to(DEV), 5, 40)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b_[0]) and torch.equal(a[1], b_[1])


@pytest.mark.parametrize("dtype,R,E,ef,k", [(torch.float16, 12, 4, 40, 5), (torch.float16, 32, 32, 64, 3),
                                            (torch.bfloat16, 32, 7, 8, 8), (torch.float32, 40, 5, 300, 10),
                                            (torch.float16, 20, 32, 3, 3), (torch.float16, 16, 2, 3000, 6),
                                            (torch.bfloat16, 32, 32, 2500, 16)])
def test_graph_several_entries_per_query(dtype, R, E, ef, k):
    """entries[B, E]: the whole batch against the oracle started from the same lists, which hold ids that
    are no nodes, repeated ids, and for some queries no usable id at all; through the plain and the
    maturity entry points (counters included), both loops (R <= 32 and R > 32), short and long lists."""
    N, B = 9000, 48
    say(f"graph multi-entry: dtype={dtype} R={R} E={E} ef={ef} k={k}")
    c = synth.make_corpus(N, 136 if dtype != torch.float32 else 132, 12, seed=61 + E, dtype=dtype, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, B)
    g = synth.ring_union(synth.knn_graph(c.x, R - 2)).contiguous()
    gen = torch.Generator().manual_seed(E)
    entries = torch.randint(-3, N + 3, (B, E), generator=gen, dtype=torch.int32)
    entries[3, :] = -1                                   # nothing usable
    entries[5, :] = entries[5, 0].clamp(0, N - 1)        # one node named E times
    if E > 1:
        entries[9, 1] = entries[9, 0]
    xd, gd, qd, ed = c.x.to(DEV), g.to(DEV), q.to(DEV), entries.to(DEV)
    ids, sc = ann.ann_graph_search_multi_typed(xd, gd, ed, qd, k, ef)
    n_ids, n_sc, stats, ema = ann.ann_graph_search_nonstall_typed(xd, gd, 0, qd, k, ef, entries=ed, tau=float("inf"))
    torch.cuda.synchronize()
    name = np_dtype_name(c.x)
    xn, qn, gn = to_np(c.x), to_np(q), g.numpy()
    o_ids, _, o_sc64, nd, ne = oracle.graph_search(xn, gn, 0, qn, k, ef, entries=entries.numpy(), dtype=name)
    assert (o_ids[3] == -1).all() and nd[3] == 0
    strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, xn, qn, dtype=name)
    say(f"  strict {strict}/{n}")
    assert strict >= n - 2
    assert torch.equal(ids, n_ids) and torch.equal(sc, n_sc)
    st = stats.cpu().numpy()
    for b in range(B):
        if (int(st[b, 1]), int(st[b, 2])) != (int(nd[b]), int(ne[b])):
            explain_divergence(xn, gn, qn, b, name, entries[b].tolist(), k, ef, o_ids[b].tolist(),
                               (int(nd[b]), int(ne[b])), n_ids[b].tolist(), (int(st[b, 1]), int(st[b, 2])))


def test_graph_several_entries_with_maturity_exit():
    """The maturity exit started from several entries: entry nodes yield no sample."""
    N, B, E, k, ef = 12_000, 64, 6, 3, 48
    c = synth.make_corpus(N, 128, 16, seed=5, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, B)
    g = synth.ring_union(synth.knn_graph(c.x.to(DEV), 14).cpu()).contiguous()
    gen = torch.Generator().manual_seed(3)
    entries = torch.randint(0, N, (B, E), generator=gen, dtype=torch.int32)
    gpu = ann.ann_graph_search_nonstall_typed(c.x.to(DEV), g.to(DEV), 0, q.to(DEV), k, ef, entries=entries.to(DEV),
                                              tau=0.8, window=60)
    torch.cuda.synchronize()
    ids, sc, stats, ema = (t.cpu().numpy() for t in gpu)
    xn, qn, gn = c.x.numpy(), q.numpy(), g.numpy()
    o = oracle.graph_search_nonstall(xn, gn, 0, qn, k, ef, tau=0.8, window=60, entries=entries.numpy())
    same = [b for b in range(B) if stats[b].tolist() == o[3][b].tolist()]
    say(f"multi-entry maturity exit: same decision {len(same)}/{B}, early exits {int(stats[:, 0].sum())}")
    assert len(same) >= B - 2 and int(stats[:, 0].sum()) >= B // 4
    compare_topk(ids[same], sc[same], o[0][same], o[2][same], xn, qn, rows=same)
    assert np.allclose(ema[same], o[4][same], rtol=5e-4, atol=5e-4)
    for b in set(range(B)) - set(same):                  # a borderline decision: the average sits at tau
        assert abs(float(ema[b]) - 0.8) < 2e-3 or abs(float(o[4][b]) - 0.8) < 2e-3, (b, ema[b], o[4][b])


def test_nan_rows_are_never_listed():
    """A corpus row of NaNs is scored and marked visited but never returned, listed or expanded,
    as an entry node, as a neighbour, in the exact search; the oracle pins the same rule."""
    N = 3000
    c = synth.make_corpus(N, 64, 6, seed=13, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 12)
    x = c.x.clone()
    bad = [5, 77, 1500]
    x[bad] = float("nan")
    g = synth.ring_union(synth.knn_graph(c.x, 10)).contiguous()
    xd, gd, qd = x.to(DEV), g.to(DEV), q.to(DEV)
    xn, qn, gn = x.numpy(), q.numpy(), g.numpy()
    for B, k in ((12, 3), (12, 10)):
        f_ids, f_sc = ann.ann_flat_search_typed(xd, qd[:B].contiguous(), k)
        torch.cuda.synchronize()
        o_ids, _, o_sc64 = oracle.flat_search(xn, qn[:B], k)
        compare_topk(f_ids.cpu().numpy(), f_sc.cpu().numpy(), o_ids, o_sc64, xn, qn[:B])
        assert not np.isin(f_ids.cpu().numpy(), bad).any()
    for entry in (5, 6):                                 # a NaN entry node, and a sound one next to it
        ids, sc = ann.ann_graph_search_typed(xd, gd, entry, qd, 4, 24)
        n_ids, _, stats, _ = ann.ann_graph_search_nonstall_typed(xd, gd, entry, qd, 4, 24, tau=float("inf"))
        torch.cuda.synchronize()
        o_ids, _, o_sc64, nd, ne = oracle.graph_search(xn, gn, entry, qn, 4, 24)
        assert np.array_equal(ids.cpu().numpy(), o_ids) and torch.equal(ids, n_ids)
        assert not np.isin(ids.cpu().numpy(), bad).any()
        if entry == 5:
            assert (o_ids == -1).all() and np.isneginf(sc.cpu().numpy()).all()
            assert stats.cpu().numpy()[:, 1:].tolist() == [[1, 0]] * 12
    e2 = torch.tensor([[5, 6]] * 12, dtype=torch.int32)
    ids, _ = ann.ann_graph_search_multi_typed(xd, gd, e2.to(DEV), qd, 4, 24)
    torch.cuda.synchronize()
    assert np.array_equal(ids.cpu().numpy(), oracle.graph_search(xn, gn, 0, qn, 4, 24, entries=e2.numpy())[0])


@pytest.mark.parametrize("N,d,C,R,dtype", [(50_000, 768, 51, 32, torch.float16), (3000, 64, 40, 32, torch.float16),
                                            (20_000, 128, 16, 20, torch.bfloat16)])
def test_graph_rows_built_by_the_library_match_the_generator(N, d, C, R, dtype):
    """k-NN rows through the library's paged exact search (R + 1 = 33 results per point, 16 per call)
    against the generator's torch matmul + top-k on the same corpus: rows identical, except where scores
    within 1e-6 of each other swap (the two sum in different orders); clusters smaller than a page and
    pools smaller than R included."""
    from paper_2505_12065_amd import graph_build
    c = synth.make_corpus(N, d, C, seed=17, sigma=(0.2, 0.5), zipf_a=1.1, dtype=dtype, device=DEV)
    got = graph_build.knn_rows_by_cluster(c.x, c.labels, c.centroids, R, 8)
    want = synth.knn_graph_cluster_restricted(c, R, 8)
    torch.cuda.synchronize()
    same = (got == want).all(dim=1)
    say(f"graph rows by the library: N={N} d={d} C={C} R={R}: identical rows {int(same.sum())}/{N}")
    assert float(same.float().mean()) >= 0.99
    xf = c.x.float()
    for i in (~same).nonzero().flatten().tolist()[:200]:
        a, b = got[i].long(), want[i].long()
        assert (a >= 0).sum() == (b >= 0).sum(), i
        sa = torch.sort((xf[a[a >= 0]] * xf[i]).sum(1)).values
        sb = torch.sort((xf[b[b >= 0]] * xf[i]).sum(1)).values
        assert torch.allclose(sa, sb, atol=2e-6), i
        assert i not in a.tolist()
    # the oracle's exact answer over the pool, for a few rows
    xn, labels = to_np(c.x), c.labels.numpy()
    cn = (c.centroids / c.centroids.norm(dim=1, keepdim=True)).numpy().astype(np.float64)
    name = np_dtype_name(c.x)
    rng = np.random.default_rng(3)
    xd = xn.view(np.uint16) if name == "bf16" else xn
    for i in rng.integers(0, N, 4).tolist():
        xi = c.x[i].float().cpu().numpy().astype(np.float64)
        near = np.argsort(-(cn @ xi), kind="stable")[:8]
        pool = np.nonzero(np.isin(labels, near))[0]
        o_ids, _, o64 = oracle.flat_search(xd[pool], xd[i:i + 1], min(R + 1, len(pool)), dtype=name)
        ref = [int(pool[j]) for j in o_ids[0] if j >= 0 and pool[j] != i][:R]
        row = [v for v in got[i].tolist() if v >= 0]
        if row != ref:
            assert sorted(row) == sorted(ref) or np.allclose(
                np.sort((c.x[row].float().cpu().numpy().astype(np.float64) @ xi)),
                np.sort((c.x[ref].float().cpu().numpy().astype(np.float64) @ xi)), atol=2e-6), i


def test_gather_ids():
    gen = torch.Generator().manual_seed(4)
    table = torch.randint(0, 1 << 30, (1000,), generator=gen, dtype=torch.int32)
    idx = torch.randint(-5, 1005, (70_001,), generator=gen, dtype=torch.int32)
    out = ann.ann_gather_ids(table.to(DEV), idx.to(DEV)).cpu()
    ok = (idx >= 0) & (idx < 1000)
    want = torch.where(ok, table[idx.clamp(0, 999).long()], torch.full_like(idx, -1))
    assert torch.equal(out, want)


def test_coarse_entries_then_graph_search_end_to_end():
    """The two-level use: exact search over one representative per cluster, row numbers turned
    into node ids, graph search from there.  Every step checked against the oracle."""
    c = synth.make_corpus(12_000, 128, 24, seed=71, dtype=torch.float16, sigma=0.3)
    q = synth.make_queries(c, 33)
    g = synth.with_reverse_edges(synth.knn_graph(c.x, 16), c.x)
    reps = synth.cluster_representatives(c)
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    rep_rows = xd[reps.long().to(DEV)].contiguous()
    cid, _ = ann.ann_flat_search_typed(rep_rows, qd, 1)
    entries = ann.ann_gather_ids(reps.to(DEV), cid.reshape(-1).contiguous())
    ids, sc = ann.ann_graph_search_entries_typed(xd, gd, entries, qd, 3, 48)
    torch.cuda.synchronize()
    xn, qn, gn = c.x.numpy(), q.numpy(), g.numpy()
    o_cid, _, _ = oracle.flat_search(xn[reps.numpy()], qn, 1)
    assert entries.cpu().numpy().tolist() == reps.numpy()[o_cid[:, 0]].tolist()
    for b in range(33):
        o_ids, _, o_sc64, _, _ = oracle.graph_search(xn, gn, int(entries[b]), qn[b:b + 1], 3, 48)
        compare_topk(ids[b:b + 1].cpu().numpy(), sc[b:b + 1].cpu().numpy(), o_ids, o_sc64, xn, qn, rows=[b])


# ------------------------------------------------------------------ configuration 2 (graph, fp16, d = 768)

@pytest.fixture(scope="module")
def cfg2_scaled():
    """Configuration 2 at a tenth of its size, graph built on the GPU by the generator module."""
    c = synth.workload_corpus(2, scale=0.1, device=DEV)
    g = synth.knn_graph_cluster_restricted(c, 32, 8)
    entry = synth.mean_entry(c.x)
    q = synth.make_queries(c, 64)
    return c, g, entry, q


@pytest.mark.parametrize("ef", [8, 16, 32, 64, 128, 256])
def test_cfg2_scaled_graph(cfg2_scaled, ef):
    c, g, entry, q = cfg2_scaled
    say(f"cfg2/10 graph: N={c.x.shape[0]} R=32 entry={entry} ef={ef} B=64 k=3")
    ids, sc = ann.ann_graph_search_typed(c.x, g, entry, q, 3, ef)
    torch.cuda.synchronize()
    xn, qn, gn = c.x.cpu().numpy(), q.cpu().numpy(), g.cpu().numpy()
    o_ids, o_sc, o_sc64, nd, ne = oracle.graph_search(xn, gn, entry, qn, 3, ef)
    strict, tolerant, n = compare_topk(ids.cpu().numpy(), sc.cpu().numpy(), o_ids, o_sc64, xn, qn)
    f_ids, _, _ = oracle.flat_search(xn, qn, 3)
    say(f"cfg2/10 ef={ef}: strict={strict}/{n} recall@3 gpu={recall(ids.cpu().numpy(), f_ids):.3f} "
        f"oracle={recall(o_ids, f_ids):.3f} n_dist={nd.mean():.0f} n_expand={ne.mean():.0f}")
    assert strict >= n - 2


# ------------------------------------------------------------------ scheduler priority levels (Section 3.2)

@pytest.mark.parametrize("n,G", [(1, 6), (5, 6), (257, 6), (3000, 6), (777, 1), (1200, 13)])
def test_priority_order_matches_oracle(n, G):
    gen = np.random.default_rng(n * 31 + G)
    R = gen.integers(0, 9, n).astype(np.int32)
    C = gen.integers(64, 8192, n).astype(np.int32)
    W = gen.random(n) * 60.0
    Wcur = np.round(gen.random(n) * 5.0, 1)                # equal queueing times occur
    if n > 10:
        W[3] = W[5]                                       # and equal metric values
    level, order = ann.ann_priority_order(torch.from_numpy(R).to(DEV), torch.from_numpy(W).to(DEV),
                                          torch.from_numpy(C).to(DEV), torch.from_numpy(Wcur).to(DEV), G)
    torch.cuda.synchronize()
    o_level, o_order = oracle.priority_order(R, W, C, Wcur, G)
    assert np.array_equal(level.cpu().numpy(), o_level)
    assert np.array_equal(order.cpu().numpy(), o_order)


def test_priority_order_with_nan_queueing_times():
    n = 700
    gen = np.random.default_rng(8)
    R = gen.integers(0, 9, n).astype(np.int32)
    C = gen.integers(100, 5000, n).astype(np.int32)
    W = gen.random(n) * 30
    Wcur = np.round(gen.random(n) * 4, 1)
    Wcur[gen.random(n) < 0.2] = np.nan
    level, order = ann.ann_priority_order(torch.from_numpy(R).to(DEV), torch.from_numpy(W).to(DEV),
                                          torch.from_numpy(C).to(DEV), torch.from_numpy(Wcur).to(DEV), 6)
    torch.cuda.synchronize()
    o_level, o_order = oracle.priority_order(R, W, C, Wcur, 6)
    assert np.array_equal(level.cpu().numpy(), o_level) and np.array_equal(order.cpu().numpy(), o_order)
    assert sorted(order.cpu().tolist()) == list(range(n))


def test_priority_order_bad_arguments():
    t = torch.zeros(4, dtype=torch.int32, device=DEV)
    w = torch.zeros(4, dtype=torch.float64, device=DEV)
    with pytest.raises(ann.AnnError):
        ann.ann_priority_order(t, w, t, w, 0)
    with pytest.raises(ValueError):
        ann.ann_priority_order(t, w.float(), t, w, 6)


# ------------------------------------------------------------------ measurement support

def test_kernel_timing_records_main_kernels():
    K = ann.binding
    c = synth.make_corpus(40_000, 128, 8, seed=3, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 200)
    g = synth.knn_graph(c.x.to(DEV), 8)
    xd, qd = c.x.to(DEV), q.to(DEV)
    ann.ann_timing_enable(True)
    for _ in range(3):
        ann.ann_flat_search_typed(xd, qd[:16].contiguous(), 3)       # streaming kernel
        ann.ann_flat_search_typed(xd, qd, 3)                         # matrix-core kernel (+ helpers, not timed)
        ann.ann_graph_search_typed(xd, g, 0, qd, 3, 16)
    ann.ann_timing_enable(False)
    ann.ann_flat_search_typed(xd, qd, 3)                             # not recorded any more
    for code, launches in ((K.KERNEL_FLAT_STREAM, 3), (K.KERNEL_FLAT_WIDE, 3), (K.KERNEL_GRAPH, 3), (K.KERNEL_FLAT_F32, 0)):
        n, ms = ann.ann_timing_read(code)
        assert n == launches and (ms > 0) == (launches > 0), (code, n, ms)
    ann.ann_timing_enable(True)                                      # switching on again drops the old records
    ann.ann_timing_enable(False)
    assert ann.ann_timing_read(K.KERNEL_GRAPH) == (0, 0.0)


def test_mfma_rate_measurement_is_plausible():
    const, rand = ann.ann_measure_mfma_rate(False, 20000), ann.ann_measure_mfma_rate(True, 20000)
    say(f"box MFMA rate: constant operands {const:.0f} TFLOP/s, random operands {rand:.0f} TFLOP/s")
    assert 500 < rand <= const * 1.05 and const < 2600
