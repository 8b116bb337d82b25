"""Host-side checks that need no GPU: the library loads, exports every function
include/ann.h declares, its constants agree with the binding, and argument errors
are rejected before anything touches a device."""
import ctypes
import os
import re

import pytest

from paper_2505_12065_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "ann.h")).read()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z0-9_]+)\s*\(", body)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert lib.ann_version() >= 100


def test_constants_match_header():
    for name in ("ANN_OK", "ANN_ERR_INVALID", "ANN_ERR_ALIGNMENT", "ANN_ERR_UNKNOWN_CORPUS", "ANN_ERR_LAUNCH",
                 "ANN_ERR_NOMEM", "ANN_F16", "ANN_BF16", "ANN_F32", "ANN_K_MAX", "ANN_EF_MAX", "ANN_R_MAX",
                 "ANN_D_MAX"):
        m = re.search(r"#define\s+%s\s+(-?\d+)" % name, HEADER)
        assert m, name
        assert int(m.group(1)) == getattr(binding, name), name


FAKE = 0x10000   # a non-null, 16-byte aligned value; never dereferenced by the checks under test


def flat(lib, corpus=FAKE, N=100, d=64, dtype=0, queries=FAKE, B=2, k=3, ids=FAKE, scores=FAKE):
    return lib.ann_flat_search_typed(corpus, N, d, dtype, queries, B, k, ids, scores, None)


def graph(lib, corpus=FAKE, N=100, d=64, dtype=0, g=FAKE, R=8, entry=0, queries=FAKE, B=2, k=3, ef=8,
          ids=FAKE, scores=FAKE):
    return lib.ann_graph_search_typed(corpus, N, d, dtype, g, R, entry, queries, B, k, ef, ids, scores, None)


def test_argument_errors_are_reported_without_a_device():
    lib = binding.lib()
    E, A = binding.ANN_ERR_INVALID, binding.ANN_ERR_ALIGNMENT
    assert flat(lib, corpus=None) == E
    assert flat(lib, queries=None) == E
    assert flat(lib, ids=None) == E
    assert flat(lib, scores=None) == E
    assert flat(lib, N=0) == E
    assert flat(lib, N=2 ** 31) == E
    assert flat(lib, B=0) == 0                      # an empty batch is a no-op, not an error
    assert flat(lib, B=-1) == E
    assert flat(lib, k=0) == E
    assert flat(lib, k=101) == E                      # k > N
    assert flat(lib, N=1000, k=binding.ANN_K_MAX + 1) == E
    assert flat(lib, dtype=7) == E
    assert flat(lib, d=binding.ANN_D_MAX + 8) == E
    assert flat(lib, d=60) == A                       # fp16 rows must be whole 16-byte chunks
    assert flat(lib, d=62, dtype=2) == A
    assert flat(lib, corpus=FAKE + 8) == A
    assert flat(lib, queries=FAKE + 2) == A
    assert b"16-byte" in lib.ann_last_error()
    assert graph(lib, g=None) == E
    assert graph(lib, R=0) == E
    assert graph(lib, R=binding.ANN_R_MAX + 1) == E
    assert graph(lib, ef=2, k=3) == E                 # ef < k is an error, not silently raised
    assert b"smaller than k" in lib.ann_last_error()
    assert graph(lib, ef=binding.ANN_EF_MAX + 1) == E
    assert graph(lib, entry=100) == E
    assert graph(lib, entry=-1) == E
    assert graph(lib, d=60) == A
    assert lib.ann_graph_search(FAKE + 64, FAKE, 8, 0, FAKE, 1, 1, 4, FAKE, FAKE, None) == binding.ANN_ERR_UNKNOWN_CORPUS
    assert lib.ann_register_corpus(None, 10, 8, 0) == E
    assert lib.ann_set_default_dtype(9) == E
    assert lib.ann_flat_workspace_bytes(1000, 64, 0, 4, 99) == E


def test_registry_round_trip():
    lib = binding.lib()
    p = FAKE + 4096
    assert lib.ann_register_corpus(p, 50, 64, 0) == 0
    # registered: the short entry point now gets past the lookup and fails on its own checks
    assert lib.ann_graph_search(p, FAKE, 8, 77, FAKE, 1, 1, 4, FAKE, FAKE, None) == binding.ANN_ERR_INVALID
    assert lib.ann_unregister_corpus(p) == 0
    assert lib.ann_graph_search(p, FAKE, 8, 0, FAKE, 1, 1, 4, FAKE, FAKE, None) == binding.ANN_ERR_UNKNOWN_CORPUS


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libann.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()
