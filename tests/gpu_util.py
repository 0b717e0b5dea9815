"""Helpers shared by the GPU parity tests: marshalling between numpy bit patterns and device tensors and
thin wrappers that call the library through its C ABI binding."""
import numpy as np
import torch

import paper_2603_04460_amd as vs
import synth

ATTN_ATOL = 2e-2      # max-abs on bf16 attention outputs (fp32 accumulation), the bar of the benchmark spec
SCORE_RTOL = 1e-3     # indexer scores, relative


def dev(bits):
    return synth.from_bits(bits, "cuda")


def bf16_to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def make_qkv(seed, hq, hkv, n, theta=1e6, local=False, rope=True):
    """Post-RoPE bf16 Q, K, V as device tensors plus their bit patterns for the oracle (same buffers)."""
    q, k, v = synth.qkv(seed, hq, hkv, n, local_structure=local)
    q, k, v = q.cuda(), k.cuda(), v.cuda()
    if rope:
        vs.rope_apply(q, 0, theta)
        vs.rope_apply(k, 0, theta)
    torch.cuda.synchronize()
    return (q, k, v), (synth.to_bits(q), synth.to_bits(k), synth.to_bits(v))


def run_sparse(q, k, v, idx_v, cnt_v, idx_s, cnt_s, want_lse=True, granularity=None):
    hq, n, _ = q.shape
    hk = k.shape[0]
    iv = torch.from_numpy(np.ascontiguousarray(idx_v, dtype=np.int32)).cuda()
    cv = torch.from_numpy(np.ascontiguousarray(cnt_v, dtype=np.int32)).cuda()
    is_ = torch.from_numpy(np.ascontiguousarray(idx_s, dtype=np.int32)).cuda()
    cs = torch.from_numpy(np.ascontiguousarray(cnt_s, dtype=np.int32)).cuda()
    ws = torch.empty(vs.sparse_prefill_workspace(hq, hk, iv.shape[0], n), dtype=torch.uint8, device="cuda")
    o = torch.full_like(q, float("nan"))
    lse = torch.full((hq, n), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    vs.sparse_prefill(q, k, v, iv, cv, is_, cs, o, lse, ws, slash_granularity=granularity)
    tiles = vs.sparse_prefill_tiles(ws)
    torch.cuda.synchronize()
    return o, lse, tiles


def run_dense(q, k, v, want_lse=True):
    hq, n, _ = q.shape
    o = torch.full_like(q, float("nan"))
    lse = torch.full((hq, n), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    vs.dense_prefill(q, k, v, o, lse)
    torch.cuda.synchronize()
    return o, lse


def lists(sets, cap=None):
    cap = cap or max(1, max(len(s) for s in sets))
    idx = np.zeros((len(sets), cap), dtype=np.int32)
    cnt = np.zeros(len(sets), dtype=np.int32)
    for h, s in enumerate(sets):
        s = sorted(int(x) for x in s)
        idx[h, :len(s)] = s
        cnt[h] = len(s)
    return idx, cnt


def check_attention(o, lse, ref_o, ref_lse, rows=None, atol=ATTN_ATOL):
    got = bf16_to_f64(o)
    if rows is not None:
        got = got[:, rows]
    assert np.isfinite(got).all()
    err = np.abs(got - ref_o).max()
    assert err <= atol, "max-abs output error %.4g" % err
    if lse is not None:
        gl = lse.cpu().numpy().astype(np.float64)
        if rows is not None:
            gl = gl[:, rows]
        fin = np.isfinite(ref_lse)
        assert np.array_equal(np.isneginf(gl), np.isneginf(ref_lse))
        lerr = np.abs(gl[fin] - ref_lse[fin]).max() if fin.any() else 0.0
        assert lerr <= 2e-3, "max-abs lse error %.4g" % lerr
    return err


def probe_values(n):
    """V for the key-set probe, [n, 128] float32 of zeros and ones (exact in bf16): channel c < 20 holds bit c of the key
    number, channel 20 + r holds 1 iff key number % 108 == r."""
    j = np.arange(n, dtype=np.int64)
    v = np.zeros((n, 128), dtype=np.float32)
    for c in range(20):
        v[:, c] = (j >> c) & 1
    v[j, 20 + (j % 108)] = 1.0
    return v


def check_key_set(k, idx_v, cnt_v, idx_s, cnt_s, hq, rows, granularity=None):
    """Decisive check of WHICH keys a sparse call kept.  With q = 0 every kept key has weight 1 / |S_i|, so
    lse[i] = ln |S_i| and o[i, c] * |S_i| is the number of kept keys whose probe channel c is one.  The oracle's kept
    count must be reproduced exactly (exp(lse) rounds to it) and every channel count exactly where it is below 100 (the
    bf16 output, 8 significant bits, then still resolves single keys: half an ulp is at most count * 2^-8 < 0.5) and
    within half an ulp, 2^-8 relative, above.  A dropped, duplicated or substituted
    key changes the count, a bit channel or two residue channels."""
    import oracle
    hk, n, _ = k.shape
    q = torch.zeros((hq, n, 128), dtype=torch.bfloat16, device="cuda")
    vp = probe_values(n)
    v = torch.from_numpy(vp).to(torch.bfloat16).cuda().unsqueeze(0).expand(hk, n, 128).contiguous()
    o, lse, _ = run_sparse(q, k, v, idx_v, cnt_v, idx_s, cnt_s, granularity=granularity)
    vb = synth.to_bits(v)
    rows = np.asarray(rows, dtype=np.int64)
    # the oracle needs q only for the scores (all zero here): a zero matrix of the right shape, K as given
    ref_o, ref_lse, live = oracle.sparse_attention(np.zeros((hq, n, 128), dtype=np.uint16), synth.to_bits(k), vb,
                                                   idx_v, cnt_v, idx_s, cnt_s, rows=rows, return_live=True,
                                                   granularity=granularity or 1)
    got_lse = lse[:, rows].cpu().numpy().astype(np.float64)
    got_o = bf16_to_f64(o[:, rows])
    empty = live == 0
    assert np.array_equal(np.isneginf(got_lse), empty)
    cnt_gpu = np.rint(np.exp(np.where(empty, 0.0, got_lse)))
    assert np.array_equal(np.where(empty, 0, cnt_gpu).astype(np.int64), live), "kept-key counts differ"
    assert np.abs(np.where(empty, 0.0, got_lse - ref_lse)).max() <= 1e-5 * max(1.0, np.log(float(live.max())))
    ref_cnt = np.rint(ref_o * live[..., None])                       # exact integers from the oracle
    got_cnt = got_o * live[..., None]
    small = ref_cnt < 100
    bad = small & (np.rint(got_cnt) != ref_cnt)
    if bad.any():
        h, r, c = [int(x[0]) for x in np.nonzero(bad)]
        raise AssertionError("kept key sets differ: head %d row %d channel %d: %.3f keys on the GPU, %d expected (|S| = %d); %d mismatches"
                             % (h, rows[r], c, got_cnt[h, r, c], ref_cnt[h, r, c], live[h, r], int(bad.sum())))
    big = ~small
    if big.any():
        assert (np.abs(got_cnt[big] - ref_cnt[big]) <= ref_cnt[big] * 2.0 ** -8 + 1e-3).all(), "kept key sets differ (large counts)"
    return live
