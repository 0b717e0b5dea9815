"""GPU parity for vs_rope_apply, vs_select_budget (bit-exact index sets) and vs_index_score (1e-3 relative),
each through the C ABI against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_04460_amd as vs
import synth

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- RoPE
@pytest.mark.parametrize("heads,n,pos0,theta,pairing", [(3, 257, 0, 1e6, 0), (2, 300, 131072 - 300, 1e6, 0),
                                                         (2, 128, 1000, 5e5, 1), (1, 1, 0, 1e4, 0)])
def test_rope_matches_oracle(heads, n, pos0, theta, pairing):
    x = synth.normal((heads, n, 128), 17 + n).to(torch.bfloat16)
    bits = synth.to_bits(x)
    y = vs.rope_apply(x.cuda(), pos0, theta, pairing)
    torch.cuda.synchronize()
    got = synth.to_bits(y)
    ref = oracle.rope_bf16(bits, pos0, theta, pairing)
    diff = got.astype(np.int32) - ref.astype(np.int32)
    # both sides round an fp64 rotation once; they may disagree only where the two fp64 libraries differ in
    # the last place next to a rounding boundary: at most one bf16 ulp, and rarely
    assert np.abs(diff).max() <= 1
    assert (diff != 0).mean() < 1e-4


# ---------------------------------------------------------------- selection
def _gpu_select(a_v, a_s, budget, use_ws=True):
    heads, n = a_v.shape
    av, as_ = torch.from_numpy(a_v).cuda(), torch.from_numpy(a_s).cuda()
    idx_v = torch.full((heads, budget.cap_v), -1, dtype=torch.int32, device="cuda")
    idx_s = torch.full((heads, budget.cap_s), -1, dtype=torch.int32, device="cuda")
    cnt_v = torch.zeros(heads, dtype=torch.int32, device="cuda")
    cnt_s = torch.zeros(heads, dtype=torch.int32, device="cuda")
    status = torch.full((heads,), 99, dtype=torch.int32, device="cuda")
    nbytes = vs.select_budget_workspace(heads, n)
    # stale contents on purpose: the library must not rely on a clean workspace
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda") if nbytes and use_ws else None
    vs.select_budget(av, as_, budget, idx_v, cnt_v, idx_s, cnt_s, status, ws)
    torch.cuda.synchronize()
    return idx_v.cpu().numpy(), cnt_v.cpu().numpy(), idx_s.cpu().numpy(), cnt_s.cpu().numpy(), status.cpu().numpy()


def _check_select(a_v, a_s, budget):
    iv, cv, is_, cs, st = _gpu_select(a_v, a_s, budget)
    n = a_v.shape[1]
    rv = oracle.select(a_v, budget.mode, budget.tau_v, budget.k_v, min(budget.n_sink, n), budget.cap_v)
    rs = oracle.select(a_s, budget.mode, budget.tau_s, budget.k_s, min(max(budget.n_local, 1), n), budget.cap_s)
    np.testing.assert_array_equal(cv, rv[1])
    np.testing.assert_array_equal(cs, rs[1])
    for h in range(a_v.shape[0]):
        np.testing.assert_array_equal(iv[h, :cv[h]], rv[0][h, :cv[h]])
        np.testing.assert_array_equal(is_[h, :cs[h]], rs[0][h, :cs[h]])
    np.testing.assert_array_equal(st, rv[2] | rs[2])
    return cv, cs


@pytest.mark.parametrize("n,tau", [(1000, 0.9), (4096, 0.5), (131072, 0.9), (70001, 0.95), (64, 1.0), (513, 0.0)])
def test_select_threshold_bit_exact(n, tau):
    a_v, a_s = synth.structured_scores(n + 1, 3, n)
    b = vs.Budget(mode=0, tau_v=tau, tau_s=tau, n_sink=4, n_local=64, cap_v=n, cap_s=n)
    b.n_sink, b.n_local = min(4, n), min(64, n)
    _check_select(a_v, a_s, b)


def test_select_ties_uniform_and_quantised():
    n = 8192
    a = np.full((2, n), 1.0 / n, dtype=np.float32)
    rng = np.random.default_rng(3)
    q = (rng.integers(1, 6, size=(2, n)) / 32768.0).astype(np.float32)        # five distinct values: massive ties
    cv, cs = _check_select(a, q, vs.Budget(mode=0, tau_v=0.9, tau_s=0.37, n_sink=0, n_local=1, cap_v=n, cap_s=n))
    assert cv.tolist() == [7373, 7373]
    _check_select(q, a, vs.Budget(mode=1, k_v=1000, k_s=n + 5, n_sink=2, n_local=3, cap_v=n, cap_s=n))


def test_select_fixed_k_and_capacity_overflow():
    n = 32768
    a_v, a_s = synth.structured_scores(9, 8, n)
    _check_select(a_v, a_s, vs.Budget(mode=1, k_v=1024, k_s=2048, n_sink=4, n_local=64, cap_v=1028, cap_s=2112))
    # capacities smaller than the pick: forced stay, best-ranked fill, overflow flagged
    iv, cv, is_, cs, st = _gpu_select(a_v, a_s, vs.Budget(mode=1, k_v=1024, k_s=2048, n_sink=4, n_local=64, cap_v=500, cap_s=100))
    assert (st & 1).all() and (cv == 500).all() and (cs == 100).all()
    _check_select(a_v, a_s, vs.Budget(mode=1, k_v=1024, k_s=2048, n_sink=4, n_local=64, cap_v=500, cap_s=100))
    _check_select(a_v, a_s, vs.Budget(mode=0, tau_v=0.9, tau_s=0.9, n_sink=4, n_local=64, cap_v=64, cap_s=65))


def test_select_bad_scores_and_errors():
    n = 300
    a = np.abs(np.random.default_rng(0).standard_normal((1, n))).astype(np.float32) / n
    a[0, 5] = np.nan; a[0, 9] = -1.0; a[0, 11] = 3.0; a[0, 13] = -0.0
    _check_select(a, a.copy(), vs.Budget(mode=0, tau_v=0.8, tau_s=0.6, n_sink=1, n_local=1, cap_v=n, cap_s=n))
    z = np.zeros((1, n), dtype=np.float32)
    _check_select(z, z, vs.Budget(mode=0, tau_v=0.9, tau_s=0.9, n_sink=2, n_local=0, cap_v=n, cap_s=n))
    with pytest.raises(vs.VsError) as e:
        _gpu_select(a, a, vs.Budget(mode=0, tau_v=1.5, tau_s=0.5, cap_v=n, cap_s=n))
    assert e.value.code == -1
    with pytest.raises(vs.VsError) as e:
        _gpu_select(a, a, vs.Budget(mode=0, tau_v=0.5, tau_s=0.5, n_sink=10, cap_v=4, cap_s=n))
    assert e.value.code == -4


def test_select_threshold_above_rounded_total():
    """tau = 1 with more than 2^13 saturated scores: the total mass (2^53 + 2^40 + 3) is not a double, ceil(tau * total)
    rounds above the total, the mass is never reached and the rule keeps everything (k = n), as the oracle does."""
    n = (1 << 13) + 1 + 3
    a = np.full((1, n), 2.0, dtype=np.float32)              # saturated: mass 2^40 each
    a[0, [100, 5000, n - 1]] = 2.0 ** -40                   # mass 1 each
    ref = oracle.select(a, 0, 1.0, 0, 0, n)
    assert ref[3][0] == n and ref[1][0] == n                # the oracle's k and count
    _check_select(a, a.copy(), vs.Budget(mode=0, tau_v=1.0, tau_s=1.0, n_sink=0, n_local=1, cap_v=n, cap_s=n))
    # and with a capacity below n: forced entries + best-ranked others, overflow flagged
    _check_select(a, a.copy(), vs.Budget(mode=0, tau_v=1.0, tau_s=1.0, n_sink=2, n_local=3, cap_v=1000, cap_s=77))


def test_select_split_over_workgroups():
    """Long problems with a workspace run the descent over one workgroup per 8192-score chunk: ties across chunk borders,
    a ragged last chunk, both rules, degenerate thresholds, bad scores, the rounded-total corner and the capacity
    overflow (redone by the single-workgroup kernel); every result equals the oracle's and the single-workgroup path's."""
    n = 40000 + 17
    assert vs.select_budget_workspace(2, n) > 0 and vs.select_budget_workspace(2, 20000) == 0
    rng = np.random.default_rng(11)
    q = (rng.integers(1, 6, size=(2, n)) / 65536.0).astype(np.float32)        # five distinct values: ties everywhere
    u = np.full((2, n), 1.0 / n, dtype=np.float32)
    a_v, a_s = synth.structured_scores(5, 2, n)
    bad = a_v.copy()
    bad[0, 5] = np.nan; bad[1, 8193] = -1.0; bad[0, 39999] = 3.0; bad[1, n - 1] = -0.0
    sat = np.full((2, n), 2.0, dtype=np.float32)
    sat[:, [100, 5000, n - 1]] = 2.0 ** -40
    cases = [
        (q, u, vs.Budget(mode=0, tau_v=0.9, tau_s=0.37, n_sink=0, n_local=1, cap_v=n, cap_s=n)),
        (q, u, vs.Budget(mode=1, k_v=12345, k_s=n + 5, n_sink=2, n_local=3, cap_v=n, cap_s=n)),
        (a_v, a_s, vs.Budget(mode=0, tau_v=1.0, tau_s=0.0, n_sink=4, n_local=64, cap_v=n, cap_s=n)),
        (a_v, a_s, vs.Budget(mode=1, k_v=0, k_s=1, n_sink=4, n_local=64, cap_v=n, cap_s=n)),
        (bad, a_s, vs.Budget(mode=0, tau_v=0.8, tau_s=0.95, n_sink=1, n_local=5000, cap_v=n, cap_s=n)),
        (sat, sat.copy(), vs.Budget(mode=0, tau_v=1.0, tau_s=1.0, n_sink=0, n_local=1, cap_v=n, cap_s=n)),
        (a_v, q, vs.Budget(mode=0, tau_v=0.9, tau_s=0.9, n_sink=4, n_local=64, cap_v=64, cap_s=5000)),      # overflow
        (np.zeros((2, n), dtype=np.float32), u, vs.Budget(mode=0, tau_v=0.9, tau_s=1.0, n_sink=2, n_local=0, cap_v=n, cap_s=n)),
    ]
    for x_v, x_s, b in cases:
        _check_select(x_v, x_s, b)
        one = _gpu_select(x_v, x_s, b, use_ws=False)
        many = _gpu_select(x_v, x_s, b, use_ws=True)
        again = _gpu_select(x_v, x_s, b, use_ws=True)           # integer atomics: the same bits whatever the order
        for r1, r2 in zip(many, again):
            np.testing.assert_array_equal(r1, r2)
        for r1, r2, cnt1 in ((one[0], many[0], one[1]), (one[2], many[2], one[3])):
            for h in range(x_v.shape[0]):
                np.testing.assert_array_equal(r1[h, :cnt1[h]], r2[h, :cnt1[h]])
        np.testing.assert_array_equal(one[1], many[1])
        np.testing.assert_array_equal(one[3], many[3])
        np.testing.assert_array_equal(one[4], many[4])


# ---------------------------------------------------------------- indexer
def _gpu_index(kb, vb, W, act, b_V=0.0, b_S=0.0):
    W_U, b_U, W_V, W_S = [torch.from_numpy(x).cuda() for x in W]
    w = vs.IndexerWeights(W_U, b_U, W_V, W_S, b_V, b_S, act)
    k, v = synth.from_bits(kb, "cuda"), synth.from_bits(vb, "cuda")
    hk, n, _ = k.shape
    a_v = torch.empty((hk, n), dtype=torch.float32, device="cuda"); a_s = torch.empty_like(a_v)
    ws = torch.empty(vs.index_score_workspace(hk, n, w.d_h), dtype=torch.uint8, device="cuda")
    vs.index_score(k, v, w, a_v, a_s, ws)
    torch.cuda.synchronize()
    return a_v.cpu().numpy().astype(np.float64), a_s.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("hk,n,d_h,act,local", [(2, 1000, 256, 1, False), (1, 4096, 256, 1, True), (2, 300, 1024, 0, False),
                                                 (1, 77, 64, 0, False), (3, 513, 128, 1, False)])
def test_indexer_scores(hk, n, d_h, act, local):
    _, k, v = synth.qkv(31 + n, 1, hk, n, local_structure=local)
    kb, vb = synth.to_bits(k), synth.to_bits(v)
    W = synth.indexer_weights(n, d_h, act)
    g_v, g_s = _gpu_index(kb, vb, W, act, 0.25, -1.5)
    r_v, r_s = oracle.index_score(kb, vb, *W, 0.25, -1.5, act=act)
    for g, r in ((g_v, r_v), (g_s, r_s)):
        rel = np.abs(g - r) / r
        assert rel.max() <= 1e-3, rel.max()
        np.testing.assert_allclose(g.sum(axis=1), 1.0, atol=1e-5)
