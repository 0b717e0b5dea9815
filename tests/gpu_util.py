"""Helpers shared by the GPU parity tests: marshalling between numpy bit patterns and device tensors and
thin wrappers that call the library through its C ABI binding."""
import numpy as np
import torch

import paper_2603_04460_amd as vs
from paper_2603_04460_amd import synth

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
