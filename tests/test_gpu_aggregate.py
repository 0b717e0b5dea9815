"""GPU parity of vs_aggregate (vertical-slash aggregation of the dense attention map and Attention Recall) against the
fp64 oracle, through the C ABI.  Tolerance: the aggregated vectors are probability distributions like the indexer's
scores, so they get the same bar (1e-3 relative, plus 1e-7 absolute for entries that are almost zero); the recall, a
single mass in [0, 1], gets 1e-4 absolute."""
import numpy as np
import pytest
import torch

import paper_2603_04460_amd as vs
import synth
from oracle import vs_oracle as oracle
from gpu_util import make_qkv, lists, run_dense

pytestmark = pytest.mark.gpu

REL, ABS, RECALL_ABS = 1e-3, 1e-7, 1e-4


def _dev_lists(iv, cv, is_, cs):
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    return f(iv), f(cv), f(is_), f(cs)


def _run(q, k, out_heads, lse=None, mask=None):
    hq, n, _ = q.shape
    hk = k.shape[0]
    index_heads = 0 if mask is None else mask[0].shape[0]
    ws = torch.empty(vs.aggregate_workspace(hq, hk, index_heads, n), dtype=torch.uint8, device="cuda")
    a_v = torch.full((out_heads, n), float("nan"), dtype=torch.float32, device="cuda")
    a_s = torch.full((out_heads, n), float("nan"), dtype=torch.float32, device="cuda")
    rec = None
    dl = None
    if mask is not None:
        rec = torch.full((out_heads,), float("nan"), dtype=torch.float32, device="cuda")
        dl = _dev_lists(*mask)
    vs.aggregate(q, k, a_v, a_s, ws, lse=lse, lists=dl, recall=rec)
    torch.cuda.synchronize()
    return (a_v.cpu().numpy().astype(np.float64), a_s.cpu().numpy().astype(np.float64),
            None if rec is None else rec.cpu().numpy().astype(np.float64))


def _oracle(qb, kb, group, mask=None):
    hq = qb.shape[0]
    av, as_, rec = [], [], []
    for h in range(hq):
        g = h // group
        if mask is None:
            a, b = oracle.vs_aggregate(qb[h], kb[g])
        else:
            iv, cv, is_, cs = mask
            ih = h if iv.shape[0] == hq else g
            a, b, r = oracle.vs_aggregate(qb[h], kb[g], idx_v=iv[ih, :cv[ih]], idx_s=is_[ih, :cs[ih]])
            rec.append(r)
        av.append(a); as_.append(b)
    return np.stack(av), np.stack(as_), np.array(rec)


def _close(got, ref):
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    bad = err > REL * np.abs(ref) + ABS
    assert not bad.any(), "worst: got %.6g ref %.6g" % (got[bad][0], ref[bad][0])


@pytest.mark.parametrize("hq,hk,n", [(1, 1, 1), (1, 1, 33), (4, 1, 64), (2, 1, 257), (8, 2, 700), (4, 4, 1000), (4, 1, 2100)])
def test_aggregate_per_query_head(hq, hk, n):
    """Ragged lengths on both sides of the 256-key workgroup and the 64-row stage; each vector sums to 1."""
    (q, k, v), (qb, kb, vb) = make_qkv(300 + n, hq, hk, n)
    a_v, a_s, _ = _run(q, k, hq)
    ref_v, ref_s, _ = _oracle(qb, kb, hq // hk)
    _close(a_v, ref_v)
    _close(a_s, ref_s)
    assert np.abs(a_v.sum(axis=1) - 1).max() < 1e-4 and np.abs(a_s.sum(axis=1) - 1).max() < 1e-4


def test_aggregate_8192_one_head_elementwise():
    """n = 8192, one head: 32 resident-key workgroups, 128 streamed stages each, the 512-entry diagonal ring wraps 16
    times and every flush window is compared, element by element, together with the recall of a mask."""
    hq, hk, n = 1, 1, 8192
    rng = np.random.default_rng(8192)
    (q, k, v), (qb, kb, vb) = make_qkv(8192, hq, hk, n, local=True)
    sv = [np.concatenate([[0, 1, 2, 3], rng.choice(np.arange(4, n), 200, replace=False)])]
    ss = [np.concatenate([np.arange(64), np.arange(3000, 3040), rng.choice(np.arange(64, n), 30, replace=False)])]
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    a_v, a_s, rec = _run(q, k, hq, mask=(iv, cv, is_, cs))
    ref_v, ref_s, ref_r = _oracle(qb, kb, 1, mask=(iv, cv, is_, cs))
    _close(a_v, ref_v)
    _close(a_s, ref_s)
    assert np.abs(rec - ref_r).max() <= RECALL_ABS, (rec, ref_r)


def test_aggregate_group_mean_and_given_lse():
    """out_heads = kv_heads gives the mean over the group's query heads; passing the normalisers of the dense attention
    call instead of recomputing them gives the same vectors."""
    hq, hk, n = 8, 2, 900
    (q, k, v), (qb, kb, vb) = make_qkv(77, hq, hk, n, local=True)
    ref_v, ref_s, _ = _oracle(qb, kb, hq // hk)
    gv = ref_v.reshape(hk, hq // hk, n).mean(axis=1)
    gs = ref_s.reshape(hk, hq // hk, n).mean(axis=1)
    a_v, a_s, _ = _run(q, k, hk)
    _close(a_v, gv)
    _close(a_s, gs)
    o, lse = run_dense(q, k, v)
    b_v, b_s, _ = _run(q, k, hq, lse=lse)
    _close(b_v, ref_v)
    _close(b_s, ref_s)


@pytest.mark.parametrize("hq,hk,n,nv,ns,per_q", [(4, 1, 600, 20, 30, False), (8, 2, 1300, 60, 40, False), (4, 2, 500, 10, 12, True)])
def test_recall_of_a_vertical_slash_mask(hq, hk, n, nv, ns, per_q):
    rng = np.random.default_rng(n)
    (q, k, v), (qb, kb, vb) = make_qkv(400 + n, hq, hk, n, local=True)
    heads = hq if per_q else hk
    sv = [np.concatenate([[0], rng.choice(np.arange(1, n), nv, replace=False)]) for _ in range(heads)]
    ss = [np.concatenate([[0], rng.choice(np.arange(1, n), ns, replace=False)]) for _ in range(heads)]
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    a_v, a_s, rec = _run(q, k, hq, mask=(iv, cv, is_, cs))
    ref_v, ref_s, ref_r = _oracle(qb, kb, hq // hk, mask=(iv, cv, is_, cs))
    _close(a_v, ref_v)
    _close(a_s, ref_s)
    assert np.abs(rec - ref_r).max() <= RECALL_ABS, (rec, ref_r)
    assert (rec > 0).all() and (rec <= 1 + 1e-5).all()


def test_recall_limits():
    """Every offset selected keeps everything (recall 1); the diagonal alone keeps exactly a_s[0]."""
    hq, hk, n = 4, 1, 400
    (q, k, v), _ = make_qkv(9, hq, hk, n)
    iv, cv = lists([[0]])
    is_, cs = lists([list(range(n))])
    _, _, rec = _run(q, k, hq, mask=(iv, cv, is_, cs))
    assert np.abs(rec - 1).max() < 1e-4
    iv, cv = lists([[]], cap=1)
    is_, cs = lists([[0]])
    _, a_s, rec = _run(q, k, hq, mask=(iv, cv, is_, cs))
    assert np.abs(rec - a_s[:, 0]).max() < 1e-5


def test_aggregate_argument_errors():
    hq, hk, n = 4, 1, 64
    (q, k, v), _ = make_qkv(1, hq, hk, n)
    a = torch.zeros((hq, n), dtype=torch.float32, device="cuda")
    ws = torch.empty(vs.aggregate_workspace(hq, hk, 0, n), dtype=torch.uint8, device="cuda")
    with pytest.raises(vs.VsError) as e:
        vs.aggregate(q, k, a, a.clone(), ws[:16])
    assert e.value.code == -3
    bad = torch.zeros((3, n), dtype=torch.float32, device="cuda")
    with pytest.raises(vs.VsError) as e:
        vs.aggregate(q, k, bad, bad.clone(), ws)
    assert e.value.code == -2
