"""The exact search through the entry point that allocates nothing (static workspace),
called through the C ABI with raw pointers, against ann_flat_search_typed on the same inputs:
ids bit-identical, scores bit-identical (same kernels, same order of operations).  Two calls
in a row, the second with a smaller input, so stale workspace contents would show."""
import ctypes
import sys

import pytest
import torch

from paper_2505_12065_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def static_call(lib, x, q, k):
    B = q.shape[0]
    ids = torch.full((B, k), -7, dtype=torch.int32, device=DEV)
    sc = torch.full((B, k), float("nan"), dtype=torch.float32, device=DEV)
    code = {torch.float16: 0, torch.bfloat16: 1, torch.float32: 2}[x.dtype]
    stream = torch.cuda.current_stream().cuda_stream
    rc = lib.ann_flat_search_static(ctypes.c_void_p(x.data_ptr()), x.shape[0], x.shape[1], code,
                                    ctypes.c_void_p(q.data_ptr()), B, k, ctypes.c_void_p(ids.data_ptr()),
                                    ctypes.c_void_p(sc.data_ptr()), ctypes.c_void_p(stream))
    return rc, ids, sc


@pytest.mark.parametrize("dtype,first,second,k", [
    (torch.float16, (60_000, 768, 300), (9_000, 768, 70), 3),     # matrix-core path, then fewer rows and queries
    (torch.float16, (60_000, 256, 16), (5_000, 256, 3), 4),       # streaming kernel
    (torch.bfloat16, (150_000, 128, 40), (140_000, 128, 9), 10),  # candidate arrays (k > 4)
    (torch.float32, (10_000, 128, 64), (700, 128, 5), 10),        # fp32 path
])
def test_static_entry_matches_allocating_entry_twice(dtype, first, second, k):
    lib = binding.lib()
    for (N, d, B) in (first, second):
        say(f"static flat: dtype={dtype} N={N} d={d} B={B} k={k}")
        c = synth.make_corpus(N, d, 16, seed=N % 97, dtype=dtype, zipf_a=None, sigma=0.3)
        q = synth.make_queries(c, B)
        xd, qd = c.x.to(DEV), q.to(DEV)
        assert binding.ann_flat_workspace_bytes(N, d, dtype, B, k) <= binding.ANN_STATIC_WORKSPACE_BYTES
        rc, ids, sc = static_call(lib, xd, qd, k)
        assert rc == binding.ANN_OK, binding.ann_last_error()
        r_ids, r_sc = binding.ann_flat_search_typed(xd, qd, k)
        torch.cuda.synchronize()
        assert torch.equal(ids, r_ids)
        assert torch.equal(sc, r_sc)


def test_static_entry_rejects_what_does_not_fit():
    lib = binding.lib()
    N, d, B, k = 200_000, 64, 2048, 10            # candidate arrays alone: 2048 x 4096 x 8 bytes
    assert binding.ann_flat_workspace_bytes(N, d, torch.float16, B, k) > binding.ANN_STATIC_WORKSPACE_BYTES
    x = torch.zeros(N, d, dtype=torch.float16, device=DEV)
    q = torch.zeros(B, d, dtype=torch.float16, device=DEV)
    rc, ids, sc = static_call(lib, x, q, k)
    torch.cuda.synchronize()
    assert rc == binding.ANN_ERR_INVALID
    assert "static" in binding.ann_last_error()
    assert bool((ids == -7).all())               # nothing was written
