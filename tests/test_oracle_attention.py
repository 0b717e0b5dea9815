"""Pins for the attention oracle (CPU only): brute force, library special case, textbook mask,
invariants and hand-worked masks.  None of them re-uses the oracle's own code."""
import os

import numpy as np
import pytest
import torch

import oracle
from brute import bits_to_f64, f32_to_bf16_bits, vs_mask, masked_attention

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_bits(rng, *shape):
    return f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def lists(*sets, cap=None):
    cap = cap or max(1, max(len(s) for s in sets))
    idx = np.zeros((len(sets), cap), dtype=np.int32)
    cnt = np.zeros(len(sets), dtype=np.int32)
    for h, s in enumerate(sets):
        s = sorted(int(x) for x in s)
        idx[h, :len(s)] = s
        cnt[h] = len(s)
    return idx, cnt


@pytest.mark.parametrize("n,d,seed", [(1, 4, 0), (2, 4, 1), (8, 8, 2), (17, 16, 3), (64, 32, 4), (33, 128, 5)])
def test_sparse_matches_dense_matrix_brute_force(n, d, seed):
    """Random lists; oracle vs the n x n mask + softmax + matmul written in numpy."""
    rng = np.random.default_rng(seed)
    hq, hk = 4, 2
    q, k, v = rand_bits(rng, hq, n, d), rand_bits(rng, hk, n, d), rand_bits(rng, hk, n, d)
    sets_v = [rng.choice(n, size=rng.integers(0, n + 1), replace=False) for _ in range(hk)]
    sets_s = [rng.choice(n, size=rng.integers(0, n + 1), replace=False) for _ in range(hk)]
    iv, cv = lists(*sets_v, cap=n)
    is_, cs = lists(*sets_s, cap=n)
    scale = 1.0 / np.sqrt(d)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, scale=scale, return_live=True)
    for h in range(hq):
        g = h // (hq // hk)
        M = vs_mask(n, sets_v[g], sets_s[g])
        ref, ref_lse = masked_attention(bits_to_f64(q[h]), bits_to_f64(k[g]), bits_to_f64(v[g]), M, scale)
        np.testing.assert_allclose(out[h], ref, rtol=0, atol=1e-12)
        fin = np.isfinite(ref_lse)
        np.testing.assert_allclose(lse[h][fin], ref_lse[fin], rtol=0, atol=1e-12)
        assert np.all(np.isneginf(lse[h][~fin]))
        np.testing.assert_array_equal(live[h], np.isfinite(M).sum(axis=1))


def test_per_query_head_index_lists():
    """index_heads == q_heads: every query head has its own lists."""
    rng = np.random.default_rng(11)
    n, d, hq, hk = 12, 8, 4, 2
    q, k, v = rand_bits(rng, hq, n, d), rand_bits(rng, hk, n, d), rand_bits(rng, hk, n, d)
    sets_v = [rng.choice(n, size=3, replace=False) for _ in range(hq)]
    sets_s = [np.concatenate([[0], rng.choice(np.arange(1, n), size=2, replace=False)]) for _ in range(hq)]
    iv, cv = lists(*sets_v)
    is_, cs = lists(*sets_s)
    out, _ = oracle.sparse_attention(q, k, v, iv, cv, is_, cs)
    for h in range(hq):
        g = h // 2
        ref, _ = masked_attention(bits_to_f64(q[h]), bits_to_f64(k[g]), bits_to_f64(v[g]),
                                  vs_mask(n, sets_v[h], sets_s[h]), 1.0 / np.sqrt(d))
        np.testing.assert_allclose(out[h], ref, atol=1e-12)


@pytest.mark.parametrize("n", [1, 5, 96, 512])
def test_dense_matches_library_sdpa(n):
    """Dense causal oracle == torch's scaled_dot_product_attention(is_causal=True) in fp64."""
    rng = np.random.default_rng(n)
    d, hq, hk = 64, 4, 2
    q, k, v = rand_bits(rng, hq, n, d), rand_bits(rng, hk, n, d), rand_bits(rng, hk, n, d)
    out, lse = oracle.dense_attention(q, k, v)
    tq = torch.from_numpy(bits_to_f64(q))
    tk = torch.from_numpy(bits_to_f64(k)).repeat_interleave(hq // hk, dim=0)
    tv = torch.from_numpy(bits_to_f64(v)).repeat_interleave(hq // hk, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    s = torch.einsum("hid,hjd->hij", tq, tk) / np.sqrt(d)
    s = s.masked_fill(torch.ones(n, n).triu(1).bool(), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), atol=1e-12)


@pytest.mark.parametrize("which", ["slash", "vertical"])
def test_full_budget_equals_dense(which):
    """All offsets (or all columns) selected => the sparse result is dense causal attention."""
    rng = np.random.default_rng(7)
    n, d = 128, 32
    q, k, v = rand_bits(rng, 2, n, d), rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d)
    full, none = list(range(n)), []
    iv, cv = lists(full if which == "vertical" else none, cap=n)
    is_, cs = lists(full if which == "slash" else none, cap=n)
    out, lse = oracle.sparse_attention(q, k, v, iv, cv, is_, cs)
    tq = torch.from_numpy(bits_to_f64(q))
    tk = torch.from_numpy(bits_to_f64(k)).expand(2, n, d)
    tv = torch.from_numpy(bits_to_f64(v)).expand(2, n, d)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
    np.testing.assert_allclose(out, ref, atol=1e-12)
    out_d, lse_d = oracle.dense_attention(q, k, v)
    np.testing.assert_allclose(out, out_d, atol=1e-13)
    np.testing.assert_allclose(lse, lse_d, atol=1e-13)


def test_sink_plus_window_mask():
    """I_v = first s columns, I_s = offsets 0..w-1 is the sink + sliding-window mask that the paper
    configures for its static baseline (Sec. "Baselines"); built here as j < s or i - j < w."""
    rng = np.random.default_rng(3)
    n, d, s, w = 48, 16, 3, 5
    q, k, v = rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d)
    iv, cv = lists(range(s))
    is_, cs = lists(range(w))
    out, _ = oracle.sparse_attention(q, k, v, iv, cv, is_, cs)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    M = np.where((j <= i) & ((j < s) | (i - j < w)), 0.0, -np.inf)
    ref, _ = masked_attention(bits_to_f64(q[0]), bits_to_f64(k[0]), bits_to_f64(v[0]), M, 1 / np.sqrt(d))
    np.testing.assert_allclose(out[0], ref, atol=1e-12)


def _read_gold(name):
    rows, I_v, I_s, n = {}, [], [], None
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.replace(":", " ").split()
        if tok[0] == "n":
            n = int(tok[1])
        elif tok[0] == "I_v":
            I_v = [int(x) for x in tok[1:]]
        elif tok[0] == "I_s":
            I_s = [int(x) for x in tok[1:]]
        elif tok[0] == "row":
            rows[int(tok[1])] = [int(x) for x in tok[2:]]
    return n, I_v, I_s, rows


@pytest.mark.parametrize("name,pairs", [("vs_mask_n8_a.txt", 19), ("vs_mask_n8_b.txt", 20)])
def test_hand_worked_masks(name, pairs):
    """With q = 0 every kept key has weight 1/|kept|, so each output row is the plain mean of V over the
    hand-listed keys; the live counts must match the hand count."""
    n, I_v, I_s, rows = _read_gold(name)
    d = 4
    q = np.zeros((1, n, d), dtype=np.uint16)
    rng = np.random.default_rng(0)
    k = rand_bits(rng, 1, n, d)
    vf = (np.arange(n)[:, None] * 1.0 + np.array([0.0, 16.0, 32.0, 64.0])[None, :]).astype(np.float32)
    v = f32_to_bf16_bits(vf)[None]                       # small integers: exact in bf16
    iv, cv = lists(I_v)
    is_, cs = lists(I_s)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True)
    assert int(live.sum()) == pairs == sum(len(r) for r in rows.values())
    for i in range(n):
        keys = rows[i]
        assert live[0, i] == len(keys)
        np.testing.assert_allclose(out[0, i], vf[keys].astype(np.float64).mean(axis=0), atol=1e-12)
        np.testing.assert_allclose(lse[0, i], np.log(len(keys)), atol=1e-12)


def test_invariants():
    rng = np.random.default_rng(5)
    n, d = 96, 16
    q, k, v = rand_bits(rng, 2, n, d), rand_bits(rng, 2, n, d), rand_bits(rng, 2, n, d)
    sv = [[0, 1, 40], [0, 7, 9, 80]]
    ss = [[0, 2, 30], [0, 1, 2, 3, 50]]
    iv, cv = lists(*sv)
    is_, cs = lists(*ss)
    # V == 1  =>  O == 1 (the kept probabilities of each row sum to one)
    ones = np.full_like(v, 0x3F80)
    out1, _ = oracle.sparse_attention(q, k, ones, iv, cv, is_, cs)
    np.testing.assert_allclose(out1, 1.0, atol=1e-13)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True)
    # live count = |{j<=i: j in I_v}| + |{o<=i: o in I_s}| - |both ways|  (set semantics, each key once)
    for h in range(2):
        for i in range(n):
            a = {j for j in sv[h] if j <= i}
            b = {i - o for o in ss[h] if o <= i}
            assert live[h, i] == len(a | b)
            assert i in (a | b)                          # the diagonal is kept (offset 0 selected)
            assert all(c in (a | b) for c in sv[h] if c <= i)   # sink / selected columns present once causal
    # an index that is already implied changes nothing: with offsets 0..n-1-c all selected, every row
    # i >= c already reaches column c through offset i - c, so adding column c to I_v is a no-op
    c = 70
    is3, cs3 = lists(list(range(n - c)), list(range(n - c)))
    out_a, _ = oracle.sparse_attention(q, k, v, iv, cv, is3, cs3)
    iv3, cv3 = lists(sorted(set(sv[0] + [c])), sorted(set(sv[1] + [c])))
    out_b, _ = oracle.sparse_attention(q, k, v, iv3, cv3, is3, cs3)
    np.testing.assert_array_equal(out_a, out_b)
    # a key outside the kept set of row i does not influence row i: perturb K and V at key 20
    k2, v2 = k.copy(), v.copy()
    k2[:, 20] = rand_bits(rng, 2, d)
    v2[:, 20] = rand_bits(rng, 2, d)
    out3, _ = oracle.sparse_attention(q, k2, v2, iv, cv, is_, cs)
    for h in range(2):
        for i in range(n):
            kept = {j for j in sv[h] if j <= i} | {i - o for o in ss[h] if o <= i}
            if 20 not in kept:
                np.testing.assert_array_equal(out3[h, i], out[h, i])
            else:
                assert not np.array_equal(out3[h, i], out[h, i])
    # causal: rows never see later keys -> truncating the sequence leaves the prefix rows unchanged
    m = 50
    ivt, cvt = lists(*[[c for c in s if c < m] for s in sv])
    ist, cst = lists(*[[o for o in s if o < m] for s in ss])
    out4, _ = oracle.sparse_attention(q[:, :m], k[:, :m], v[:, :m], ivt, cvt, ist, cst)
    np.testing.assert_array_equal(out4, out[:, :m])


def test_row_subset_and_empty_rows():
    rng = np.random.default_rng(9)
    n, d = 40, 8
    q, k, v = rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d)
    iv, cv = lists([5])
    is_, cs = lists([3])                                   # no offset 0: rows 0..2 have no key at all
    out, lse = oracle.sparse_attention(q, k, v, iv, cv, is_, cs)
    assert np.all(out[0, :3] == 0) and np.all(np.isneginf(lse[0, :3]))
    rows = np.array([39, 0, 7, 7, 12])
    out_r, lse_r = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, rows=rows)
    np.testing.assert_array_equal(out_r[0], out[0, rows])
    np.testing.assert_array_equal(lse_r[0], lse[0, rows])


def test_vs_aggregate_and_recall():
    """Column / diagonal sums of the causal attention matrix (Sec. "Obtaining Ground Truth") each total n
    before the division by n; recall (Eq. R(S)) of the full mask is 1 and matches a numpy evaluation."""
    rng = np.random.default_rng(21)
    n, d = 24, 8
    q, k = rand_bits(rng, n, d), rand_bits(rng, n, d)
    a_v, a_s = oracle.vs_aggregate(q, k)
    np.testing.assert_allclose(a_v.sum(), 1.0, atol=1e-13)
    np.testing.assert_allclose(a_s.sum(), 1.0, atol=1e-13)
    S = bits_to_f64(q) @ bits_to_f64(k).T / np.sqrt(d)
    S[np.triu_indices(n, 1)] = -np.inf
    A = np.exp(S - S.max(axis=1, keepdims=True))
    A /= A.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(a_v, A.sum(axis=0) / n, atol=1e-13)
    np.testing.assert_allclose(a_s, [np.trace(A, -o) / n for o in range(n)], atol=1e-13)
    I_v, I_s = [0, 9], [0, 1, 6]
    _, _, rec = oracle.vs_aggregate(q, k, idx_v=I_v, idx_s=I_s)
    keep = np.isfinite(vs_mask(n, I_v, I_s))
    np.testing.assert_allclose(rec, (A * keep).sum() / n, atol=1e-13)
    _, _, rec_full = oracle.vs_aggregate(q, k, idx_v=[], idx_s=list(range(n)))
    np.testing.assert_allclose(rec_full, 1.0, atol=1e-13)


def _granular_mask(n, I_v, I_s, g):
    """The tile-granular kept set from its range form (numpy, no oracle code): with b = g * floor(i / g) the first row of
    the aligned block of i, offset o reaches the keys b - o .. b + g - 1 - o (rows past the end of the sequence reach
    nothing); a selected column is kept as in the exact mask; then causality."""
    M = np.full((n, n), -np.inf)
    for i in range(n):
        b = g * (i // g)
        last_row = min(b + g, n) - 1
        for o in I_s:
            lo, hi = max(b - int(o), 0), min(last_row - int(o), i)
            if lo <= hi:
                M[i, lo:hi + 1] = 0.0
        for c in I_v:
            if int(c) <= i:
                M[i, int(c)] = 0.0
    return M


def _window_mask(n, I_s, g, forward):
    """Two MISREADINGS of "the block of row i", for contrast with the aligned blocks: a sliding window of the g rows
    ending at i (forward = False) or starting at i (forward = True)."""
    M = np.zeros((n, n), dtype=bool)
    for i in range(n):
        block = range(i, min(i + g, n)) if forward else range(max(i - g + 1, 0), i + 1)
        for j in range(i + 1):
            M[i, j] = any((r - j) in I_s for r in block)
    return M


def test_tile_granular_hand_worked_example():
    """n = 8, g = 4: the example whose tile-granular mask happens to be the dense causal mask."""
    n, I_v, I_s, rows = _read_gold("vs_mask_n8_g4.txt")
    d = 4
    q = np.zeros((1, n, d), dtype=np.uint16)
    k = rand_bits(np.random.default_rng(1), 1, n, d)
    vf = (np.arange(n)[:, None] + np.array([0.0, 16.0, 32.0, 64.0])[None, :]).astype(np.float32)
    v = f32_to_bf16_bits(vf)[None]
    iv, cv = lists(I_v)
    is_, cs = lists(I_s)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, granularity=4)
    assert int(live.sum()) == 36
    for i in range(n):
        assert live[0, i] == len(rows[i]) == i + 1
        np.testing.assert_allclose(out[0, i], vf[rows[i]].astype(np.float64).mean(axis=0), atol=1e-12)
    dense, _ = oracle.dense_attention(q, k, v)
    np.testing.assert_allclose(out, dense, atol=1e-13)


def test_tile_granular_hand_worked_example_aligned_blocks():
    """n = 12, g = 4, I_s = {0, 6}, no columns: the hand-listed rows separate aligned blocks (54 live pairs) from a
    trailing window (60), a forward window (36), the exact mask (18) and the dense mask (78).  q = 0, so every output
    row is the plain mean of V over the hand-listed keys."""
    n, I_v, I_s, rows = _read_gold("vs_mask_n12_g4.txt")
    assert (n, I_v, I_s) == (12, [], [0, 6])
    d = 4
    q = np.zeros((1, n, d), dtype=np.uint16)
    k = rand_bits(np.random.default_rng(2), 1, n, d)
    vf = (np.arange(n)[:, None] + np.array([0.0, 16.0, 32.0, 64.0])[None, :]).astype(np.float32)
    v = f32_to_bf16_bits(vf)[None]
    iv, cv = lists(I_v, cap=1)
    is_, cs = lists(I_s)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, granularity=4)
    assert sum(len(r) for r in rows.values()) == 54 == int(live.sum())
    for i in range(n):
        assert live[0, i] == len(rows[i])
        np.testing.assert_allclose(out[0, i], vf[rows[i]].astype(np.float64).mean(axis=0), atol=1e-12)
        np.testing.assert_allclose(lse[0, i], np.log(len(rows[i])), atol=1e-12)
    # the fixture agrees with the range form, and the competing readings really differ on this example
    kept = np.isfinite(_granular_mask(n, I_v, I_s, 4))
    assert all(sorted(np.flatnonzero(kept[i]).tolist()) == rows[i] for i in range(n))
    assert int(_window_mask(n, set(I_s), 4, forward=False).sum()) == 60
    assert int(_window_mask(n, set(I_s), 4, forward=True).sum()) == 36
    assert int(np.isfinite(vs_mask(n, I_v, I_s)).sum()) == 18
    exact, _, live1 = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, granularity=1)
    assert int(live1.sum()) == 18


@pytest.mark.parametrize("n,g,seed", [(24, 4, 0), (40, 8, 1), (70, 32, 2), (33, 32, 3), (16, 1, 4)])
def test_tile_granular_matches_definition_and_contains_exact(n, g, seed):
    rng = np.random.default_rng(seed)
    d = 8
    q, k, v = rand_bits(rng, 2, n, d), rand_bits(rng, 1, n, d), rand_bits(rng, 1, n, d)
    sv = rng.choice(n, size=3, replace=False)
    ss = np.concatenate([[0], rng.choice(np.arange(1, n), size=4, replace=False)])
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, granularity=g)
    M = _granular_mask(n, sv, ss, g)
    for h in range(2):
        ref, _ = masked_attention(bits_to_f64(q[h]), bits_to_f64(k[0]), bits_to_f64(v[0]), M, 1 / np.sqrt(d))
        np.testing.assert_allclose(out[h], ref, atol=1e-12)
    exact = np.isfinite(vs_mask(n, sv, ss))
    assert np.all(np.isfinite(M)[exact])                     # superset of the element-exact mask
    if g == 1:
        assert np.array_equal(np.isfinite(M), exact)


# ---------------------------------------------------------------- chunked prefill (query rows at positions pos0 ..)
@pytest.mark.parametrize("name,pos0", [("vs_mask_n8_a.txt", 5), ("vs_mask_n8_b.txt", 3), ("vs_mask_n8_a.txt", 0)])
def test_chunk_hand_worked_split(name, pos0):
    """The hand-worked 8-token examples, split: the chunk holding positions pos0 .. 7 must keep, for each of its rows,
    exactly the keys the fixture lists for that position (q = 0: the output is the mean of V over them)."""
    n, I_v, I_s, rows = _read_gold(name)
    d = 4
    k = rand_bits(np.random.default_rng(0), 1, n, d)
    vf = (np.arange(n)[:, None] * 1.0 + np.array([0.0, 16.0, 32.0, 64.0])[None, :]).astype(np.float32)
    v = f32_to_bf16_bits(vf)[None]
    q = np.zeros((1, n - pos0, d), dtype=np.uint16)
    iv, cv = lists(I_v)
    is_, cs = lists(I_s)
    out, lse, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, pos0=pos0)
    assert out.shape == (1, n - pos0, d)
    for r in range(n - pos0):
        keys = rows[pos0 + r]
        assert live[0, r] == len(keys)
        np.testing.assert_allclose(out[0, r], vf[keys].astype(np.float64).mean(axis=0), atol=1e-12)
        np.testing.assert_allclose(lse[0, r], np.log(len(keys)), atol=1e-12)


def test_chunk_aligned_blocks_of_absolute_positions():
    """Tile-granular chunk: blocks are aligned in absolute positions, so a chunk that starts inside a block (pos0 = 6, g = 4)
    keeps for positions 6 and 7 what the fixture lists for them (their block is {4..7}, offset 6 reaches keys 0 and 1)."""
    n, I_v, I_s, rows = _read_gold("vs_mask_n12_g4.txt")
    d, pos0 = 4, 6
    k = rand_bits(np.random.default_rng(3), 1, n, d)
    vf = (np.arange(n)[:, None] + np.array([0.0, 16.0, 32.0, 64.0])[None, :]).astype(np.float32)
    v = f32_to_bf16_bits(vf)[None]
    q = np.zeros((1, n - pos0, d), dtype=np.uint16)
    iv, cv = lists(I_v, cap=1)
    is_, cs = lists(I_s)
    out, _, live = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, return_live=True, granularity=4, pos0=pos0)
    for r in range(n - pos0):
        assert live[0, r] == len(rows[pos0 + r])
        np.testing.assert_allclose(out[0, r], vf[rows[pos0 + r]].astype(np.float64).mean(axis=0), atol=1e-12)


@pytest.mark.parametrize("g", [1, 4])
def test_chunks_equal_full_call_and_brute_force(g):
    """Any split of a sequence into chunks reproduces the rows of the full call (same arithmetic per row: identical);
    a chunk also matches the numpy mask written for its absolute positions; keys past the chunk's last position do not
    matter."""
    rng = np.random.default_rng(40 + g)
    n, d, hq, hk = 50, 8, 4, 2
    q, k, v = rand_bits(rng, hq, n, d), rand_bits(rng, hk, n, d), rand_bits(rng, hk, n, d)
    sv = [rng.choice(n, size=5, replace=False) for _ in range(hk)]
    ss = [np.concatenate([[0], rng.choice(np.arange(1, n), size=6, replace=False)]) for _ in range(hk)]
    iv, cv = lists(*sv)
    is_, cs = lists(*ss)
    full, full_lse = oracle.sparse_attention(q, k, v, iv, cv, is_, cs, granularity=g)
    dfull, dfull_lse = oracle.dense_attention(q, k, v)
    for bounds in ([0, 13, 32, 50], [0, 49, 50], [0, 50]):
        if g > 1 and any(b % g for b in bounds[:-1]):
            continue                                       # a chunk boundary inside a block changes which positions exist
        for a, b in zip(bounds[:-1], bounds[1:]):
            out, lse = oracle.sparse_attention(q[:, a:b], k, v, iv, cv, is_, cs, granularity=g, pos0=a) if g == 1 else \
                oracle.sparse_attention(q[:, a:b], k[:, :b], v[:, :b], iv, cv, is_, cs, granularity=g, pos0=a)
            if g == 1 or b == n:
                np.testing.assert_array_equal(out, full[:, a:b])
                np.testing.assert_array_equal(lse, full_lse[:, a:b])
            do, dl = oracle.dense_attention(q[:, a:b], k, v, pos0=a)
            np.testing.assert_array_equal(do, dfull[:, a:b])
            np.testing.assert_array_equal(dl, dfull_lse[:, a:b])
    # brute force for one chunk, written for absolute positions
    a, b = 13, 32
    out, lse = oracle.sparse_attention(q[:, a:b], k, v, iv, cv, is_, cs, granularity=g, pos0=a)
    for h in range(hq):
        gk = h // (hq // hk)
        M = _granular_mask(b, sv[gk], ss[gk], g)[a:b]      # the sequence ends at the chunk's last position
        Mfull = np.full((b - a, n), -np.inf)
        Mfull[:, :b] = M
        P = bits_to_f64(q[h, a:b]) @ bits_to_f64(k[gk]).T / np.sqrt(d) + Mfull       # [chunk rows, all keys]
        mx = P.max(axis=1, keepdims=True)
        E = np.exp(P - mx)
        np.testing.assert_allclose(out[h], (E / E.sum(axis=1, keepdims=True)) @ bits_to_f64(v[gk]), atol=1e-12)
        np.testing.assert_allclose(lse[h], mx[:, 0] + np.log(E.sum(axis=1)), atol=1e-12)
