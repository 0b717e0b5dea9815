"""GPU parity of chunked prefill (query rows at positions pos0 .., vs_sparse_prefill_chunk / vs_dense_prefill_chunk), of
batches folded into the head dimension, and of the list validator, through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_04460_amd as vs
import synth
from gpu_util import make_qkv, lists, check_attention, bf16_to_f64, probe_values

pytestmark = pytest.mark.gpu


def _dev_lists(*arrs):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda() for a in arrs]


def _sets(rng, n, heads, nv, ns):
    sv = [np.unique(np.concatenate([[0], rng.choice(n, size=nv, replace=False)])) for _ in range(heads)]
    ss = []
    for _ in range(heads):
        offs = {0, 1, 2}
        while len(offs) < ns:
            start = int(rng.integers(0, n))
            offs.update(range(start, min(n, start + int(rng.integers(1, 30)))))
        ss.append(sorted(offs))
    return sv, ss


def _run_chunk(q, k, v, dl, pos0, n_q, gran=None, dense=False):
    hq = q.shape[0]
    qc = q[:, pos0:pos0 + n_q].contiguous()
    o = torch.full_like(qc, float("nan"))
    lse = torch.full((hq, n_q), float("nan"), dtype=torch.float32, device="cuda")
    if dense:
        vs.dense_prefill(qc, k, v, o, lse, pos0=pos0)
    else:
        ws = torch.empty(vs.sparse_prefill_workspace(hq, k.shape[0], dl[0].shape[0], k.shape[1]), dtype=torch.uint8, device="cuda")
        vs.sparse_prefill(qc, k, v, *dl, o, lse, ws, slash_granularity=gran, pos0=pos0)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("hq,hk,n_kv,pos0,n_q,gran,per_q", [
    (8, 2, 1500, 700, 800, None, False),     # second half, aligned start
    (8, 2, 1500, 701, 333, None, False),     # unaligned start, chunk ends before the last key
    (4, 1, 1000, 999, 1, None, False),       # a single decode-like row at the end
    (4, 4, 900, 77, 500, None, False),       # G = 1 (128-row tiles), unaligned
    (4, 2, 900, 331, 569, None, False),      # G = 2
    (8, 2, 700, 45, 600, None, True),        # one list per query head
    (8, 2, 1500, 704, 796, 32, False),       # tile-granular, aligned start
    (4, 1, 5000, 4097, 903, None, False),    # several gather stages, unaligned
])
def test_sparse_chunk_matches_oracle(hq, hk, n_kv, pos0, n_q, gran, per_q):
    rng = np.random.default_rng(n_kv + pos0)
    (q, k, v), (qb, kb, vb) = make_qkv(800 + n_kv, hq, hk, n_kv)
    ih = hq if per_q else hk
    sv, ss = _sets(rng, n_kv, ih, n_kv // 12, n_kv // 10)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    dl = _dev_lists(iv, cv, is_, cs)
    o, lse = _run_chunk(q, k, v, dl, pos0, n_q, gran)
    ref_o, ref_lse = oracle.sparse_attention(qb[:, pos0:pos0 + n_q], kb, vb, iv, cv, is_, cs, granularity=gran or 1, pos0=pos0)
    check_attention(o, lse, ref_o, ref_lse)
    if gran is None:
        # key-set probe on the chunk: q = 0, probe V
        vp = torch.from_numpy(probe_values(n_kv)).to(torch.bfloat16).cuda().unsqueeze(0).expand(hk, n_kv, 128).contiguous()
        qz = torch.zeros_like(q)
        o2, lse2 = _run_chunk(qz, k, vp, dl, pos0, n_q)
        r_o, r_lse, live = oracle.sparse_attention(np.zeros((hq, n_q, 128), dtype=np.uint16), kb, synth.to_bits(vp), iv, cv, is_,
                                                   cs, return_live=True, pos0=pos0)
        assert np.array_equal(np.rint(np.exp(lse2.cpu().numpy().astype(np.float64))).astype(np.int64), live)
        cnt = np.rint(r_o * live[..., None])
        got = bf16_to_f64(o2) * live[..., None]
        small = cnt < 100
        assert np.array_equal(np.rint(got[small]), cnt[small])


def test_chunks_stitch_to_the_full_call():
    """Three chunks (unaligned boundaries) against one call on the whole sequence: same rows up to summation order."""
    hq, hk, n = 8, 2, 3000
    rng = np.random.default_rng(4)
    (q, k, v), (qb, kb, vb) = make_qkv(4321, hq, hk, n)
    sv, ss = _sets(rng, n, hk, 200, 250)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    dl = _dev_lists(iv, cv, is_, cs)
    full_o, full_lse = _run_chunk(q, k, v, dl, 0, n)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs)
    check_attention(full_o, full_lse, ref_o, ref_lse)
    for a, b in ((0, 1111), (1111, 2049), (2049, 3000)):
        # a chunk sees only the keys that exist when it runs
        o, lse = _run_chunk(q[:, :b].contiguous(), k[:, :b].contiguous(), v[:, :b].contiguous(), dl_clip(dl, b), a, b - a)
        assert np.abs(bf16_to_f64(o) - bf16_to_f64(full_o[:, a:b])).max() <= 1e-2
        assert (lse - full_lse[:, a:b]).abs().max().item() <= 2e-3
        check_attention(o, lse, ref_o[:, a:b], ref_lse[:, a:b])


def dl_clip(dl, n):
    """Lists restricted to entries < n (a chunk call takes columns and offsets in [0, n_kv))."""
    out = []
    for idx, cnt in ((dl[0], dl[1]), (dl[2], dl[3])):
        i, c = idx.cpu().numpy(), cnt.cpu().numpy()
        sets = [[int(x) for x in i[h, :c[h]] if x < n] for h in range(i.shape[0])]
        a, b = lists(sets, cap=i.shape[1])
        out += _dev_lists(a, b)
    return out


@pytest.mark.parametrize("hq,hk,n_kv,pos0,n_q", [(8, 2, 1200, 600, 600), (4, 1, 777, 333, 444), (4, 4, 500, 499, 1), (16, 2, 640, 129, 300)])
def test_dense_chunk_matches_oracle(hq, hk, n_kv, pos0, n_q):
    (q, k, v), (qb, kb, vb) = make_qkv(900 + n_kv, hq, hk, n_kv)
    o, lse = _run_chunk(q, k, v, None, pos0, n_q, dense=True)
    ref_o, ref_lse = oracle.dense_attention(qb[:, pos0:pos0 + n_q], kb, vb, pos0=pos0)
    check_attention(o, lse, ref_o, ref_lse)


def test_chunk_argument_errors():
    (q, k, v), _ = make_qkv(1, 4, 1, 128)
    z = torch.zeros((1, 4), dtype=torch.int32, device="cuda"); c = torch.ones(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(vs.sparse_prefill_workspace(4, 1, 1, 128), dtype=torch.uint8, device="cuda")
    qc = q[:, :64].contiguous()
    o = torch.empty_like(qc)
    with pytest.raises(vs.VsError) as e:
        vs.sparse_prefill(qc, k, v, z, c, z, c, o, None, ws, pos0=65)          # runs past the keys
    assert e.value.code == -1
    with pytest.raises(vs.VsError) as e:
        vs.sparse_prefill(qc, k, v, z, c, z, c, o, None, ws, pos0=33, slash_granularity=32)
    assert e.value.code == -2
    with pytest.raises(vs.VsError) as e:
        vs.dense_prefill(qc, k, v, o, pos0=-1)
    assert e.value.code == -1


@pytest.mark.parametrize("batch,hq,hk,n", [(3, 8, 2, 700), (20, 4, 2, 300)])
def test_batch_folded_into_heads(batch, hq, hk, n):
    """A batch of sequences is batch * heads heads in the same layout (20 x 2 = 40 KV heads: more work queues than the
    32 of one layer).  Each sequence has its own lists; the batched call must equal the per-sequence calls bit for bit
    and the oracle."""
    rng = np.random.default_rng(batch)
    (q, k, v), (qb, kb, vb) = make_qkv(50 + batch, batch * hq, batch * hk, n)
    sv, ss = _sets(rng, n, batch * hk, 40, 60)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    dl = _dev_lists(iv, cv, is_, cs)
    o, lse = _run_chunk(q, k, v, dl, 0, n)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs)
    check_attention(o, lse, ref_o, ref_lse)
    for b in (0, batch - 1):
        sl_q, sl_k = slice(b * hq, (b + 1) * hq), slice(b * hk, (b + 1) * hk)
        one = [t[sl_k].contiguous() for t in dl]
        o1, lse1 = _run_chunk(q[sl_q].contiguous(), k[sl_k].contiguous(), v[sl_k].contiguous(), one, 0, n)
        assert torch.equal(o1.view(torch.int16), o[sl_q].view(torch.int16)) and torch.equal(lse1, lse[sl_q])
    # the other stages take the folded batch as it is: scores and selection per (sequence, head)
    W = synth.indexer_weights(5, 64, 1)
    wd = vs.IndexerWeights(*[torch.from_numpy(x).cuda() for x in W], 0.0, 0.0, 1)
    a_v = torch.empty((batch * hk, n), dtype=torch.float32, device="cuda"); a_s = torch.empty_like(a_v)
    ws = torch.empty(vs.index_score_workspace(batch * hk, n, 64), dtype=torch.uint8, device="cuda")
    vs.index_score(k, v, wd, a_v, a_s, ws)
    torch.cuda.synchronize()
    r_v, r_s = oracle.index_score(kb[:2], vb[:2], *W, act=1)
    assert (np.abs(a_v[:2].cpu().numpy() - r_v) / r_v).max() <= 1e-3 and (np.abs(a_s[:2].cpu().numpy() - r_s) / r_s).max() <= 1e-3


def test_validate_lists():
    n, cap = 500, 8
    idx = np.array([[0, 3, 9, 100, 499, 0, 0, 0],      # fine, 5 entries
                    [0, 3, 3, 100, 0, 0, 0, 0],        # duplicate
                    [5, 4, 9, 0, 0, 0, 0, 0],          # unsorted
                    [-2, 3, 9, 500, 0, 0, 0, 0],       # out of range at both ends (legal: ignored by the kernels)
                    [1, 2, 3, 4, 5, 6, 7, 8],          # count larger than the capacity
                    [7, 0, 0, 0, 0, 0, 0, 0]], dtype=np.int32)   # empty list
    cnt = np.array([5, 4, 3, 4, 9, 0], dtype=np.int32)
    report = torch.full((6,), -1, dtype=torch.int32, device="cuda")
    vs.validate_lists(torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(), n, report)
    torch.cuda.synchronize()
    assert report.cpu().tolist() == [0, 4, 4, 2, 1, 0]
