"""The largest supported sequence (n = 2^20, VS_MAX_SEQ) through every entry point, one query head and one KV head, in
the launch configuration the library chooses itself.  The oracle checks sampled outputs it can compute one by one
(rows of the attention calls, the whole selection, the whole indexer at a small hidden width); the aggregation, whose
definition is O(n^2) for the oracle, is checked through properties that hold at any size."""
import numpy as np
import pytest
import torch

import paper_2603_04460_amd as vs
import synth
from oracle import vs_oracle as oracle
from gpu_util import make_qkv, lists, run_sparse, run_dense, check_attention, check_key_set

pytestmark = pytest.mark.gpu

N = 1 << 20


@pytest.fixture(scope="module")
def qkv():
    return make_qkv(2020, 1, 1, N, theta=1e6)


def test_sparse_attention_max_n(qkv):
    """32768 key blocks: the touched-block words fill their LDS table (1024 words), late tiles list several hundred
    blocks and gather a few hundred columns."""
    (q, k, v), (qb, kb, vb) = qkv
    rng = np.random.default_rng(11)
    cols = np.unique(np.concatenate([np.arange(4), rng.choice(N, 300, replace=False)]))
    offs = np.unique(np.concatenate([np.arange(64), rng.choice(N, 12, replace=False),
                                     np.arange(500000, 500000 + 700), np.arange(N - 40, N)]))
    iv, cv = lists([cols])
    is_, cs = lists([offs])
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    rows = synth.sample_rows(3, N, 40, 40, 48)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)
    assert tiles > 0
    # which keys were kept, exactly (the values above average hundreds of keys)
    check_key_set(k, iv, cv, is_, cs, 1, rows)
    check_key_set(k, iv, cv, is_, cs, 1, rows, granularity=32)


def test_dense_attention_max_n(qkv):
    (q, k, v), (qb, kb, vb) = qkv
    o, lse = run_dense(q, k, v)
    rows = synth.sample_rows(4, N, 16, 32, 16)
    ref_o, ref_lse = oracle.dense_attention(qb, kb, vb, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_indexer_and_selection_max_n(qkv):
    (q, k, v), (qb, kb, vb) = qkv
    d_h = 64
    W = synth.indexer_weights(77, d_h, 1)
    wd = vs.IndexerWeights(*[torch.from_numpy(x).cuda() for x in W], 0.0, 0.0, 1)
    ws = torch.empty(vs.index_score_workspace(1, N, d_h), dtype=torch.uint8, device="cuda")
    a_v = torch.empty((1, N), dtype=torch.float32, device="cuda")
    a_s = torch.empty_like(a_v)
    vs.index_score(k, v, wd, a_v, a_s, ws)
    torch.cuda.synchronize()
    ref_v, ref_s = oracle.index_score(kb, vb, *W, act=1)
    for got, ref in ((a_v, ref_v), (a_s, ref_s)):
        g = got.cpu().numpy().astype(np.float64)
        assert np.abs(g - ref).max() <= 1e-3 * np.abs(ref).max() and (np.abs(g - ref) <= 1e-3 * ref + 1e-12).all()
    # selection of the GPU's own scores: bit-exact against the oracle fed the same fp32 values
    cap = N // 4
    b = vs.Budget(0, 0.9, 0.9, 0, 0, 4, 64, cap, cap)
    idx_v = torch.empty((1, cap), dtype=torch.int32, device="cuda"); idx_s = torch.empty_like(idx_v)
    cnt_v = torch.empty(1, dtype=torch.int32, device="cuda"); cnt_s = torch.empty_like(cnt_v)
    status = torch.empty(1, dtype=torch.int32, device="cuda")
    refs = [oracle.select(scores.cpu().numpy(), 0, 0.9, 0, forced, cap) for scores, forced in ((a_v, 4), (a_s, 64))]
    # without a workspace (one workgroup per problem) and with one (128 chunks per problem)
    for wsel in (None, torch.empty(vs.select_budget_workspace(1, N), dtype=torch.uint8, device="cuda")):
        idx_v.fill_(-1); idx_s.fill_(-1)
        vs.select_budget(a_v, a_s, b, idx_v, cnt_v, idx_s, cnt_s, status, wsel)
        torch.cuda.synchronize()
        for (ri, rc, _, _), idx, cnt in zip(refs, (idx_v, idx_s), (cnt_v, cnt_s)):
            c = int(cnt.item())
            assert c == int(rc[0])
            assert np.array_equal(idx[0, :c].cpu().numpy(), ri[0, :c])


def test_aggregate_properties_max_n(qkv):
    """Each vector sums to 1; with every offset selected the recall is 1; with the diagonal alone it is a_s[0]."""
    (q, k, v), _ = qkv
    ws = torch.empty(vs.aggregate_workspace(1, 1, 1, N), dtype=torch.uint8, device="cuda")
    a_v = torch.empty((1, N), dtype=torch.float32, device="cuda"); a_s = torch.empty_like(a_v)
    rec = torch.empty(1, dtype=torch.float32, device="cuda")
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    iv, cv = lists([[0]]); is_, cs = lists([[0]])
    vs.aggregate(q, k, a_v, a_s, ws, lists=(f(iv), f(cv), f(is_), f(cs)), recall=rec)
    torch.cuda.synchronize()
    assert abs(a_v.double().sum().item() - 1) < 1e-3 and abs(a_s.double().sum().item() - 1) < 1e-3
    assert (a_v >= 0).all() and (a_s >= 0).all()
    # column 0 and the diagonal: kept mass = a_v[0] + a_s[0] - A[0,0]/n (the pair (0,0) is in both)
    expect = a_v[0, 0].item() + a_s[0, 0].item() - 1.0 / N
    assert abs(rec.item() - expect) < 1e-5
