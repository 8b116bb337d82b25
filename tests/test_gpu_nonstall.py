"""GPU parity of the graph search with the maturity (non-stall) exit of Section 3.3 /
Appendix B.2 against the CPU oracle, through the C ABI.

The exit decision compares a binary32 moving average with tau on both sides, but the
scores that feed it are summed in a different order (fp32 on the GPU, fp64 rounded to
fp32 in the oracle), so a query whose average passes within rounding distance of tau may
leave one expansion earlier or later.  Such a query is still checked: the GPU result must
be exactly what the oracle holds when it is cut after the GPU's number of expansions."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_12065_amd as ann
from paper_2505_12065_amd import synth
from parity import compare_nonstall, np_dtype_name, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def run_both(x, g, entry, q, k, ef, tau, window, ready=None):
    """x, g, q: cpu tensors.  GPU (ids, scores, stats, ema) as numpy and the oracle's tuple."""
    ids, sc, stats, ema = ann.ann_graph_search_nonstall_typed(x.to(DEV), g.to(DEV), entry, q.to(DEV), k, ef, tau=tau,
                                                              window=window, engine_ready=ready)
    torch.cuda.synchronize()
    o = oracle.graph_search_nonstall(to_np(x), g.numpy(), entry, to_np(q), k, ef, tau=tau, window=window,
                                     dtype=np_dtype_name(x))
    return ids.cpu().numpy(), sc.cpu().numpy(), stats.cpu().numpy(), ema.cpu().numpy(), o


def check_against_oracle(x, g, entry, q, k, ef, tau, window, gpu, o, max_off=None):
    return compare_nonstall(gpu, o, to_np(x), g.numpy(), to_np(q), np_dtype_name(x), entry, k, ef, tau, window, max_off)


@pytest.fixture(scope="module")
def small():
    c = synth.make_corpus(20_000, 128, 16, seed=77, dtype=torch.float16, zipf_a=None, sigma=0.3)
    q = synth.make_queries(c, 96)
    g = synth.ring_union(synth.knn_graph(c.x.to(DEV), 15).cpu()).contiguous()
    return c, q, g


@pytest.mark.parametrize("ef,tau,window", [(32, 0.9, 500), (64, 0.8, 100), (64, 0.6, 30), (128, 0.9, 200),
                                           (16, 0.5, 10), (256, 0.95, 500),
                                           (64, 6.0, 500), (64, 10.0, 500),    # these two: early and natural stops mixed
                                           (2500, 0.9, 500), (3000, 1.5, 300)])   # two-level list
def test_nonstall_matches_oracle(small, ef, tau, window):
    c, q, g = small
    say(f"non-stall: N=20000 R={g.shape[1]} ef={ef} tau={tau} window={window}")
    *gpu, o = run_both(c.x, g, 5, q, 3, ef, tau, window)
    n_same, n_off = check_against_oracle(c.x, g, 5, q, 3, ef, tau, window, gpu, o)
    say(f"  identical decisions {n_same}/{n_same + n_off}; early exits gpu={int(gpu[2][:, 0].sum())} "
        f"oracle={int(o[3][:, 0].sum())}; mean expansions {gpu[2][:, 2].mean():.1f}")


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
@pytest.mark.parametrize("R", [7, 33, 70])
def test_nonstall_dtypes_and_wide_rows(dtype, R):
    """Rows longer than one scoring pass, junk and repeated ids in the rows."""
    N, d = 6000, 136 if dtype != torch.float32 else 132
    c = synth.make_corpus(N, d, 8, seed=R, dtype=dtype, zipf_a=None, sigma=0.4)
    q = synth.make_queries(c, 24)
    gen = torch.Generator().manual_seed(R)
    near = synth.knn_graph(c.x, max(1, R // 2))
    rnd = torch.randint(-1, N + 3, (N, R - near.shape[1]), generator=gen, dtype=torch.int32)
    g = torch.cat([near, rnd], 1).contiguous()
    g[:, -1] = g[:, 0]                            # every row names its first neighbour twice
    say(f"non-stall rows: dtype={dtype} R={R}")
    *gpu, o = run_both(c.x, g, 3, q, 4, 48, 0.7, 60)
    check_against_oracle(c.x, g, 3, q, 4, 48, 0.7, 60, gpu, o, max_off=2)
    *again, _ = run_both(c.x, g, 3, q, 4, 48, 0.7, 60)            # which slot scores a repeated id may vary:
    for u, v in zip(gpu, again):                                    # the outputs may not
        assert np.array_equal(u, v)


def test_nonstall_never_mature_equals_plain_search_and_counts_are_exact(small):
    """tau = +inf: ids and scores are those of the plain entry point bit for bit, and the
    scored-node / expansion counts are the oracle's, which shows that no node is scored twice."""
    c, q, g = small
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    for ef in (8, 64, 200):
        ids, sc, stats, ema = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, ef, tau=float("inf"), window=500)
        p_ids, p_sc = ann.ann_graph_search_typed(xd, gd, 5, qd, 3, ef)
        torch.cuda.synchronize()
        assert torch.equal(ids, p_ids) and torch.equal(sc, p_sc)
        _, _, _, nd, ne = oracle.graph_search(c.x.numpy(), g.numpy(), 5, q.numpy(), 3, ef)
        st = stats.cpu().numpy()
        assert (st[:, 0] == 0).all()
        assert np.array_equal(st[:, 1], nd) and np.array_equal(st[:, 2], ne), ef


def test_engine_ready_word(small):
    """Engine not ready: mature queries keep searching to the natural stop.  Ready: as with
    no word at all.  The word may live in device memory or in pinned host memory."""
    c, q, g = small
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    free = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=0.6, window=30)
    plain = ann.ann_graph_search_typed(xd, gd, 5, qd, 3, 64)
    torch.cuda.synchronize()
    assert int(free[2][:, 0].sum()) > 0
    for make in (lambda v: torch.tensor([v], dtype=torch.int32, device=DEV),
                 lambda v: torch.tensor([v], dtype=torch.int32).pin_memory()):
        busy = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=0.6, window=30, engine_ready=make(0))
        torch.cuda.synchronize()
        assert int(busy[2][:, 0].sum()) == 0
        assert torch.equal(busy[0], plain[0]) and torch.equal(busy[1], plain[1])
        ready = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=0.6, window=30, engine_ready=make(1))
        torch.cuda.synchronize()
        for a, b in zip(ready, free):
            assert torch.equal(a, b)


def test_nonstall_repeated_calls_and_smaller_batch(small):
    """The visited workspace is cleared by every call: a second call and a call on fewer
    queries give the same rows."""
    c, q, g = small
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    a = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=0.8, window=100)
    b = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=0.8, window=100)
    s = ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd[:17].contiguous(), 3, 64, tau=0.8, window=100)
    torch.cuda.synchronize()
    for u, v, w in zip(a, b, s):
        assert torch.equal(u, v) and torch.equal(u[:17], w)
    assert ann.ann_graph_nonstall_workspace_bytes(20_000, 96) == 96 * 64 * 40      # one bit per node, in 64-byte units


def test_nonstall_bad_arguments(small):
    c, q, g = small
    xd, gd, qd = c.x.to(DEV), g.to(DEV), q.to(DEV)
    with pytest.raises(ann.AnnError) as e:
        ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, window=0)
    assert e.value.code == -1
    with pytest.raises(ann.AnnError):
        ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 64, tau=float("nan"))
    with pytest.raises(ann.AnnError):
        ann.ann_graph_search_nonstall_typed(xd, gd, 5, qd, 3, 2)      # ef < k
