"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (no GPU is touched by these calls)."""
import ctypes
import os
import re

import pytest

import paper_2603_04460_amd as vs
from paper_2603_04460_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "vsprefill.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vs_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(vs.library_path())
    names = header_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names
    assert vs.version().startswith("vsprefill")


def test_strerror_and_workspace_queries():
    L = binding._load()
    assert L.vs_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.vs_strerror(code) not in (b"ok", b"unknown status")
    assert vs.sparse_prefill_workspace(32, 8, 8, 131072) > 3 * 8 * 131072 // 8 // 2
    assert vs.sparse_prefill_workspace(32, 8, 5, 131072) == 0          # index_heads must be q_heads or kv_heads
    # two bf16 halves of W_U + one (max, sum) pair per head, direction and block of 64 tokens
    assert vs.index_score_workspace(8, 131072, 256) == 2 * 256 * 256 * 2 + 8 * 2 * 2048 * 8
    # wider layers also hold the partial logits of every slice of 256 hidden units
    assert vs.index_score_workspace(8, 131072, 1024) == 2 * 1024 * 256 * 2 + 8 * 2 * 2048 * 8 + 2 * 4 * 8 * 131072 * 4
    assert vs.index_train_workspace(8, 4096, 256) > vs.index_score_workspace(8, 4096, 256)
    assert vs.index_score_workspace(8, 131072, 100) == 0               # d_h must be a multiple of 64
    # short problems need none (one workgroup each, everything in LDS); long ones: three histograms of 4096 (mass, count)
    # per problem, the redo flags, four descent states per problem and three counts per 8192-score chunk
    assert vs.select_budget_workspace(8, 20000) == 0
    assert vs.select_budget_workspace(8, 131072) == 3 * 16 * 4096 * 12 + 256 + 16 * 4 * 48 + 16 * 16 * 3 * 4


def test_host_side_argument_checks():
    L = binding._load()
    buf = (ctypes.c_char * 4096)()
    p = ctypes.addressof(buf)
    p = (p + 15) & ~15
    vp = ctypes.c_void_p
    # null pointers, bad sizes, misalignment -> INVALID_ARG; unsupported head ratio / length -> UNSUPPORTED
    assert L.vs_dense_prefill(None, vp(p), vp(p), 4, 1, 64, 0.1, vp(p), None, None) == -1
    assert L.vs_dense_prefill(vp(p + 4), vp(p), vp(p), 4, 1, 64, 0.1, vp(p), None, None) == -1
    assert L.vs_dense_prefill(vp(p), vp(p), vp(p), 4, 1, 0, 0.1, vp(p), None, None) == -1
    assert L.vs_dense_prefill(vp(p), vp(p), vp(p), 4, 1, 64, -1.0, vp(p), None, None) == -1
    assert L.vs_dense_prefill(vp(p), vp(p), vp(p), 4, 3, 64, 0.1, vp(p), None, None) == -2
    assert L.vs_dense_prefill(vp(p), vp(p), vp(p), 4, 1, (1 << 20) + 1, 0.1, vp(p), None, None) == -2
    assert L.vs_sparse_prefill(vp(p), vp(p), vp(p), 4, 1, 64, 0.1, vp(p), vp(p), 4, vp(p), vp(p), 4, 1,
                               vp(p), None, None, 0, None) == -3      # workspace missing
    assert L.vs_sparse_prefill(vp(p), vp(p), vp(p), 4, 1, 64, 0.1, vp(p), vp(p), 4, vp(p), vp(p), 4, 2,
                               vp(p), None, vp(p), 1 << 20, None) == -1   # index_heads neither q_heads nor kv_heads
    assert L.vs_rope_apply(vp(p), 2, 16, 0, 0.5, 0, None) == -1        # theta base must exceed 1
    assert L.vs_rope_apply(vp(p), 2, 16, 0, 1e6, 3, None) == -1
    b = binding._Budget(0, 1.5, 0.5, 0, 0, 0, 1, 8, 8)
    assert L.vs_select_budget(vp(p), vp(p), 1, 64, ctypes.byref(b), vp(p), vp(p), vp(p), vp(p), None, None, 0, None) == -1
    b = binding._Budget(0, 0.5, 0.5, 0, 0, 9, 1, 8, 8)                 # 9 forced sinks do not fit a capacity of 8
    assert L.vs_select_budget(vp(p), vp(p), 1, 64, ctypes.byref(b), vp(p), vp(p), vp(p), vp(p), None, None, 0, None) == -4
    b = binding._Budget(2, 0.5, 0.5, 0, 0, 0, 1, 8, 8)
    assert L.vs_select_budget(vp(p), vp(p), 1, 64, ctypes.byref(b), vp(p), vp(p), vp(p), vp(p), None, None, 0, None) == -1
    # long problem with a workspace that is too small / misaligned: refused on the host, before any launch
    b = binding._Budget(0, 0.5, 0.5, 0, 0, 0, 1, 8, 8)
    assert L.vs_select_budget(vp(p), vp(p), 1, 65536, ctypes.byref(b), vp(p), vp(p), vp(p), vp(p), None, vp(p), 1024, None) == -3
    assert L.vs_select_budget(vp(p), vp(p), 1, 65536, ctypes.byref(b), vp(p), vp(p), vp(p), vp(p), None, vp(p + 4), 1 << 24, None) == -1
    w = binding._Indexer(p, p, p, p, 0.0, 0.0, 100, 1)
    assert L.vs_index_score(vp(p), vp(p), 1, 64, ctypes.byref(w), vp(p), vp(p), vp(p), 1 << 20, None) == -2
    w = binding._Indexer(p, p, p, p, 0.0, 0.0, 256, 7)
    assert L.vs_index_score(vp(p), vp(p), 1, 64, ctypes.byref(w), vp(p), vp(p), vp(p), 1 << 20, None) == -1
    w = binding._Indexer(p, p, p, p, 0.0, 0.0, 256, 1)
    assert L.vs_index_score(vp(p), vp(p), 1, 64, ctypes.byref(w), vp(p), vp(p), vp(p), 16, None) == -3
    # vs_aggregate(q, k, q_heads, kv_heads, n, scale, lse, out_heads, a_v, a_s, idx_v, cnt_v, cap_v, idx_s, cnt_s, cap_s,
    #              index_heads, recall, ws, ws_bytes, stream)
    agg = lambda *a: L.vs_aggregate(*a)
    big = 1 << 20
    assert agg(None, vp(p), 4, 1, 64, 0.1, None, 4, vp(p), vp(p), None, None, 0, None, None, 0, 0, None, vp(p), big, None) == -1
    assert agg(vp(p), vp(p), 4, 3, 64, 0.1, None, 4, vp(p), vp(p), None, None, 0, None, None, 0, 0, None, vp(p), big, None) == -2
    assert agg(vp(p), vp(p), 4, 1, 64, 0.1, None, 2, vp(p), vp(p), None, None, 0, None, None, 0, 0, None, vp(p), big, None) == -2
    assert agg(vp(p), vp(p), 4, 1, 64, 0.1, None, 4, vp(p), vp(p), None, None, 0, None, None, 0, 0, None, vp(p), 64, None) == -3
    # a recall needs the lists
    assert agg(vp(p), vp(p), 4, 1, 64, 0.1, None, 4, vp(p), vp(p), None, None, 0, None, None, 0, 1, vp(p), vp(p), big, None) == -1
    assert vs.aggregate_workspace(32, 8, 8, 131072) >= 32 * 131072 * 4
    assert vs.aggregate_workspace(32, 8, 0, 131072) == 32 * 131072 * 4


def test_product_path_does_not_import_the_oracle():
    """The package and the benchmark's timed path must not reach into oracle/ (only tests, smoke() and the
    cpu_baseline leg may)."""
    pkg = os.path.join(ROOT, "paper_2603_04460_amd")
    imp = re.compile(r"^\s*(import|from)\s+oracle\b|vs_oracle|libvs_oracle", re.M)
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            assert not imp.search(open(os.path.join(pkg, name)).read()), name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert not imp.search(open(os.path.join(pkg, "csrc", name)).read()), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    head, _, tail = bench.partition("def cpu_baseline")
    assert "import oracle" not in head
    assert "import oracle" not in tail.partition("def main")[2]


def test_synth_generators_are_seeded_and_shaped():
    import numpy as np
    import synth
    q1, k1, v1 = synth.qkv(7, 8, 2, 256, local_structure=True)
    q2, k2, v2 = synth.qkv(7, 8, 2, 256, local_structure=True)
    assert q1.shape == (8, 256, 128) and k1.shape == (2, 256, 128)
    assert np.array_equal(synth.to_bits(k1), synth.to_bits(k2)) and np.array_equal(synth.to_bits(q1), synth.to_bits(q2))
    kk = k1.float().numpy()
    c1 = np.mean(kk[:, 1:] * kk[:, :-1])                 # neighbouring tokens are correlated ...
    c40 = np.mean(kk[:, 40:] * kk[:, :-40])              # ... tokens further apart than the window are not
    assert c1 > 0.8 and abs(c40) < 0.1
    iv, cv, is_, cs = synth.fixed_lists(3, 4096)
    assert iv.shape == (1, 64) and is_.shape == (1, 128) and iv[0, :4].tolist() == [0, 1, 2, 3]
    assert np.all(np.diff(iv[0]) > 0) and np.all(np.diff(is_[0]) > 0) and is_[0, 63] == 63
    a_v, a_s = synth.structured_scores(1, 2, 1024)
    assert abs(a_v.sum(axis=1) - 1).max() < 1e-5 and abs(a_s.sum(axis=1) - 1).max() < 1e-5
    rows = synth.sample_rows(0, 1000, 8, 8, 16)
    assert rows[0] == 0 and rows[-1] == 999 and len(rows) <= 32
