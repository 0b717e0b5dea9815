"""GPU parity: vs_dense_prefill and vs_sparse_prefill (through the C ABI) against the fp64 oracle,
element by element on the same post-RoPE bf16 buffers.  Tolerance: max-abs 2e-2 on the bf16 outputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_04460_amd as vs
import synth
from gpu_util import make_qkv, run_sparse, run_dense, lists, check_attention, check_key_set, bf16_to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("hq,hk,n", [(4, 1, 200), (1, 1, 1000), (2, 1, 300), (8, 1, 257), (8, 2, 64), (3, 1, 130),
                                     (4, 1, 1), (4, 1, 31), (4, 1, 33), (4, 1, 63), (4, 1, 64), (4, 1, 65), (4, 1, 127),
                                     (4, 1, 129), (2, 2, 191), (1, 1, 511), (6, 2, 320), (16, 2, 700)])
def test_dense_small(hq, hk, n):
    (q, k, v), (qb, kb, vb) = make_qkv(100 + n, hq, hk, n)
    o, lse = run_dense(q, k, v)
    ref_o, ref_lse = oracle.dense_attention(qb, kb, vb)
    check_attention(o, lse, ref_o, ref_lse)


def test_config1_single_head_4096_fixed_lists():
    """Single head, n = 4096, columns {0..3} + 60 random, offsets {0..63} + 64 random; every row checked."""
    n = 4096
    seed = synth.config_seed(1)
    (q, k, v), (qb, kb, vb) = make_qkv(seed, 1, 1, n)
    iv, cv, is_, cs = synth.fixed_lists(seed, n)
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    ref_o, ref_lse, live = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, return_live=True)
    check_attention(o, lse, ref_o, ref_lse)
    assert live.sum() / 1024 <= tiles <= (n // 32) * (n // 32 + 1) // 2
    # same call twice: bit-identical (no float atomics on the result path)
    o2, lse2, tiles2 = run_sparse(q, k, v, iv, cv, is_, cs)
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16)) and torch.equal(lse, lse2) and tiles == tiles2


def _random_sets(rng, n, heads, nv, ns, runs=True):
    sv, ss = [], []
    for _ in range(heads):
        cols = set(rng.choice(n, size=min(nv, n), replace=False).tolist())
        offs = {0}
        while len(offs) < min(ns, n):
            start = int(rng.integers(0, n))
            length = int(rng.integers(1, 40)) if runs else 1
            offs.update(range(start, min(n, start + length)))
        sv.append(cols)
        ss.append(offs)
    return sv, ss


@pytest.mark.parametrize("hq,hk,n,nv,ns,per_q", [
    (8, 2, 1500, 100, 200, False),     # ragged n, GQA 4, runs + scattered columns (in-block and gathered)
    (4, 1, 777, 300, 5, False),        # many columns, few diagonals -> gather dominated
    (4, 4, 640, 20, 60, False),        # G = 1: 256-row tiles
    (4, 2, 900, 50, 100, False),       # G = 2
    (8, 2, 700, 40, 80, True),         # one list per query head
    (40, 40, 200, 10, 20, False),      # more KV heads (work queues) than the 32 of one layer
    (80, 40, 150, 8, 12, False),       # the same with two query heads per KV head
    (16, 2, 500, 30, 50, False),       # G = 8: two workgroups per tile
])
def test_sparse_random_lists(hq, hk, n, nv, ns, per_q):
    rng = np.random.default_rng(n)
    (q, k, v), (qb, kb, vb) = make_qkv(200 + n, hq, hk, n)
    ih = hq if per_q else hk
    sv, ss = _random_sets(rng, n, ih, nv, ns)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    ref_o, ref_lse, live = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, return_live=True)
    check_attention(o, lse, ref_o, ref_lse)
    assert tiles * 1024 >= live.sum()


def test_sparse_randomized_sweep():
    """36 seeded random cases in one process: lengths 1 .. 2600 (ragged against every tile size), head layouts with
    group sizes 1, 2, 4 and 8, list sizes from empty to a third of the sequence, scattered and run-shaped offsets, with
    and without the diagonal, exact and tile-granular mode, per-KV-head and per-query-head lists."""
    rng = np.random.default_rng(20260304)
    layouts = [(1, 1), (2, 1), (4, 1), (4, 2), (8, 2), (8, 1), (4, 4)]
    for case in range(36):
        hq, hk = layouts[int(rng.integers(len(layouts)))]
        n = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 255, 256, 257, 500, 1000, 1023, 1025, 1777, 2600]))
        per_q = bool(rng.integers(2)) and hq != hk
        ih = hq if per_q else hk
        nv = int(rng.integers(0, max(1, n // 3) + 1))
        ns = int(rng.integers(0, max(1, n // 6) + 1))
        runs = bool(rng.integers(2))
        gran = 32 if rng.integers(3) == 0 else None
        sv, ss = [], []
        for _ in range(ih):
            cols = set(rng.choice(n, size=min(nv, n), replace=False).tolist()) if nv else set()
            offs = set() if rng.integers(4) == 0 else {0}
            guard = 0
            while len(offs) < min(ns, n) and guard < 10000:
                start = int(rng.integers(0, n))
                length = int(rng.integers(1, 40)) if runs else 1
                offs.update(range(start, min(n, start + length)))
                guard += 1
            sv.append(cols)
            ss.append(offs)
        iv, cv = lists(sv)
        is_, cs = lists(ss)
        (q, k, v), (qb, kb, vb) = make_qkv(5000 + case, hq, hk, n)
        o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs, granularity=gran)
        ref_o, ref_lse, live = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, return_live=True, granularity=gran or 1)
        try:
            check_attention(o, lse, ref_o, ref_lse)
            assert tiles * 1024 >= live.sum()
        except AssertionError as e:
            raise AssertionError("case %d: heads %d/%d n %d nv %d ns %d runs %s per_q %s g %s: %s"
                                 % (case, hq, hk, n, nv, ns, runs, per_q, gran, e))


def test_workspace_reused_across_calls_of_different_size():
    """One oversized workspace, a large call, then a small one, then the large one again: every call re-initialises
    the counters and bitmaps it uses, so results do not depend on what the workspace held before."""
    rng = np.random.default_rng(99)
    hq, hk = 8, 2
    ws = torch.empty(vs.sparse_prefill_workspace(hq, hk, hk, 4096) + 4096, dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)
    outs = []
    for n in (1500, 300, 1500):
        (q, k, v), (qb, kb, vb) = make_qkv(600 + n, hq, hk, n)
        sv, ss = _random_sets(np.random.default_rng(n), n, hk, 60, 90)
        iv, cv = lists(sv)
        is_, cs = lists(ss)
        f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
        o = torch.full_like(q, float("nan"))
        lse = torch.full((hq, n), float("nan"), dtype=torch.float32, device="cuda")
        vs.sparse_prefill(q, k, v, f(iv), f(cv), f(is_), f(cs), o, lse, ws)
        torch.cuda.synchronize()
        ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs)
        check_attention(o, lse, ref_o, ref_lse)
        outs.append(o.clone())
    assert torch.equal(outs[0].view(torch.int16), outs[2].view(torch.int16))


def test_sparse_edge_cases():
    n, hq, hk = 300, 4, 1
    (q, k, v), (qb, kb, vb) = make_qkv(7, hq, hk, n)
    cases = {
        "diagonal only": ([[]], [[0]]),
        "columns only, no diagonal: rows before the first column are empty": ([[5, 70, 299]], [[]]),
        "offset without the diagonal": ([[]], [[3]]),
        "all offsets = dense": ([[]], [list(range(n))]),
        "all columns = dense": ([list(range(n))], [[]]),
        "far offset only touches late rows": ([[0]], [[0, 290]]),
        "column in the last block": ([[298]], [[0, 1]]),
    }
    for name, (sv, ss) in cases.items():
        iv, cv = lists(sv, cap=n)
        is_, cs = lists(ss, cap=n)
        o, lse, _ = run_sparse(q, k, v, iv, cv, is_, cs)
        ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs)
        check_attention(o, lse, ref_o, ref_lse)
    # full budget == the dense kernel's own answer to within rounding of different tile orders
    iv, cv = lists([[]], cap=4)
    is_, cs = lists([list(range(n))])
    o, _, _ = run_sparse(q, k, v, iv, cv, is_, cs)
    od, _ = run_dense(q, k, v)
    assert np.abs(bf16_to_f64(o) - bf16_to_f64(od)).max() <= 1e-2
    # out-of-range and negative entries are ignored
    iv = np.array([[-5, 3, 9, n, n + 7]], dtype=np.int32); cv = np.array([5], dtype=np.int32)
    is_ = np.array([[0, 2, n + 1]], dtype=np.int32); cs = np.array([3], dtype=np.int32)
    o, lse, _ = run_sparse(q, k, v, iv, cv, is_, cs)
    iv2, cv2 = lists([[3, 9]]); is2, cs2 = lists([[0, 2]])
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv2, cv2, is2, cs2)
    check_attention(o, lse, ref_o, ref_lse)


def test_sparse_many_tiles_sampled_rows():
    """n = 16384, 8 / 2 heads: several hundred tiles per row block, more gathered columns than one gather list holds
    (several gather rounds), checked on a declared row sample."""
    n, hq, hk = 16384, 8, 2
    rng = np.random.default_rng(5)
    (q, k, v), (qb, kb, vb) = make_qkv(55, hq, hk, n)
    sv, ss = _random_sets(rng, n, hk, 6000, 700)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    rows = synth.sample_rows(5, n, 48, 48, 64)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_sparse_several_gather_rounds():
    """Two slash offsets and 9000 selected columns at n = 16384: late query tiles gather almost all of them, several
    times what one gather list holds (at most 2304 entries), so the kernel runs several gather rounds per tile."""
    n, hq, hk = 16384, 4, 1
    rng = np.random.default_rng(17)
    (q, k, v), (qb, kb, vb) = make_qkv(57, hq, hk, n)
    iv, cv = lists([rng.choice(n, size=9000, replace=False)])
    is_, cs = lists([[0, 1]])
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    rows = synth.sample_rows(17, n, 40, 72, 48)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_sparse_several_block_rounds():
    """Every 16th offset selected at n = 36000: every 32-key block is crossed by a selected diagonal, so late query
    tiles list many more blocks (1125) than one block list holds (128): several block rounds per tile."""
    n, hq, hk = 36000, 4, 1
    (q, k, v), (qb, kb, vb) = make_qkv(58, hq, hk, n)
    iv, cv = lists([[0, 5, 17000]])
    is_, cs = lists([list(range(0, n, 16))])
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    rows = synth.sample_rows(18, n, 32, 96, 32)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_sparse_long_sequence_class():
    """n = 140000 (> 131072): the kernel size with 1024 words of touched-block bits and the shorter gather list, with a
    4:1 group, a few thousand columns (several gather rounds late in the sequence) and banded offsets."""
    n, hq, hk = 140000, 4, 1
    rng = np.random.default_rng(23)
    (q, k, v), (qb, kb, vb) = make_qkv(59, hq, hk, n)
    cols = np.unique(np.concatenate([np.arange(4), rng.choice(n, size=4000, replace=False)]))
    offs = np.unique(np.concatenate([np.arange(48), np.arange(70000, 70090), rng.choice(n, size=20, replace=False)]))
    iv, cv = lists([cols])
    is_, cs = lists([offs])
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs)
    rows = synth.sample_rows(19, n, 40, 40, 48)
    ref_o, ref_lse = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_dense_sampled_rows_8192():
    n, hq, hk = 8192, 8, 2
    (q, k, v), (qb, kb, vb) = make_qkv(66, hq, hk, n)
    o, lse = run_dense(q, k, v)
    rows = synth.sample_rows(6, n, 32, 32, 32)
    ref_o, ref_lse = oracle.dense_attention(qb, kb, vb, rows=rows)
    check_attention(o, lse, ref_o, ref_lse, rows=rows)


def test_argument_errors():
    (q, k, v), _ = make_qkv(1, 4, 1, 64)
    o = torch.empty_like(q)
    iv = torch.zeros((1, 4), dtype=torch.int32, device="cuda"); cv = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(vs.sparse_prefill_workspace(4, 1, 1, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(vs.VsError) as e:
        vs.sparse_prefill(q, k, v, iv, cv, iv, cv, o, None, ws[:16])
    assert e.value.code == -3
    with pytest.raises(vs.VsError) as e:
        vs.dense_prefill(q[:3].contiguous(), torch.cat([k, k]), torch.cat([v, v]), o[:3].contiguous())
    assert e.value.code == -2
    with pytest.raises(vs.VsError) as e:
        vs.dense_prefill(q, k, v, o, scale=-1.0)
    assert e.value.code == -1


@pytest.mark.parametrize("hq,hk,n,nv,ns", [(8, 2, 1500, 100, 200), (4, 1, 777, 30, 40), (4, 4, 640, 20, 60), (4, 1, 33, 2, 3)])
def test_tile_granular_slash_mode(hq, hk, n, nv, ns):
    """vs_sparse_prefill_tiled with g = 32 against the oracle's tile-granular mask; g = 1 equals vs_sparse_prefill."""
    rng = np.random.default_rng(n + 1)
    (q, k, v), (qb, kb, vb) = make_qkv(300 + n, hq, hk, n)
    sv, ss = _random_sets(rng, n, hk, nv, ns)
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    o, lse, tiles = run_sparse(q, k, v, iv, cv, is_, cs, granularity=32)
    ref_o, ref_lse, live = oracle.sparse_attention(qb, kb, vb, iv, cv, is_, cs, return_live=True, granularity=32)
    check_attention(o, lse, ref_o, ref_lse)
    assert tiles * 1024 >= live.sum()
    o1, lse1, _ = run_sparse(q, k, v, iv, cv, is_, cs, granularity=1)
    o0, lse0, _ = run_sparse(q, k, v, iv, cv, is_, cs)
    assert torch.equal(o1.view(torch.int16), o0.view(torch.int16)) and torch.equal(lse1, lse0)
    ws = torch.empty(vs.sparse_prefill_workspace(hq, hk, hk, n), dtype=torch.uint8, device="cuda")
    with pytest.raises(vs.VsError) as e:
        vs.sparse_prefill(q, k, v, torch.from_numpy(iv).cuda(), torch.from_numpy(cv).cuda(), torch.from_numpy(is_).cuda(),
                          torch.from_numpy(cs).cuda(), o, None, ws, slash_granularity=16)
    assert e.value.code == -2


def _long_case(name):
    """The list recipes of the long-sequence tests above: (n, hq, hk, column sets, offset sets, row sample)."""
    if name == "gather_rounds":
        n = 16384
        cols = [np.random.default_rng(17).choice(n, size=9000, replace=False)]
        return n, 4, 1, cols, [[0, 1]], synth.sample_rows(17, n, 40, 72, 48)
    if name == "block_rounds":
        n = 36000
        return n, 4, 1, [[0, 5, 17000]], [list(range(0, n, 16))], synth.sample_rows(18, n, 32, 96, 32)
    if name == "long_class":
        n = 140000
        rng = np.random.default_rng(23)
        cols = np.unique(np.concatenate([np.arange(4), rng.choice(n, size=4000, replace=False)]))
        offs = np.unique(np.concatenate([np.arange(48), np.arange(70000, 70090), rng.choice(n, size=20, replace=False)]))
        return n, 4, 1, [cols], [offs], synth.sample_rows(19, n, 40, 40, 48)
    if name == "many_tiles":
        n = 16384
        sv, ss = _random_sets(np.random.default_rng(5), n, 2, 6000, 700)
        return n, 8, 2, sv, ss, synth.sample_rows(5, n, 48, 48, 64)
    raise KeyError(name)


@pytest.mark.parametrize("name,gran", [("gather_rounds", None), ("block_rounds", None), ("long_class", None),
                                       ("many_tiles", None), ("many_tiles", 32), ("long_class", 32)])
def test_key_sets_long_sequences(name, gran):
    """Exact kept-key sets (count, bit channels, residue channels) of the multi-round / long-sequence cases: the value
    tests above average thousands of keys and cannot see a single wrong key."""
    n, hq, hk, sv, ss, rows = _long_case(name)
    k = synth.qkv(900 + n, hq, hk, n)[1].cuda()
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    live = check_key_set(k, iv, cv, is_, cs, hq, rows, granularity=gran)
    assert live.max() > 1000


def test_key_sets_small_random():
    """The same probe on 24 small random cases (every head layout, per-query-head lists, both granularities), all rows."""
    rng = np.random.default_rng(777)
    layouts = [(1, 1), (2, 1), (4, 1), (4, 2), (8, 2), (8, 1), (4, 4)]
    for case in range(24):
        hq, hk = layouts[int(rng.integers(len(layouts)))]
        n = int(rng.choice([1, 33, 64, 255, 257, 500, 1000, 1025, 1777, 2600]))
        per_q = bool(rng.integers(2)) and hq != hk
        ih = hq if per_q else hk
        sv, ss = _random_sets(rng, n, ih, int(rng.integers(0, n // 3 + 1)), int(rng.integers(1, n // 6 + 2)), runs=bool(rng.integers(2)))
        gran = 32 if rng.integers(3) == 0 else None
        iv, cv = lists(sv)
        is_, cs = lists(ss)
        k = synth.qkv(7000 + case, hq, hk, n)[1].cuda()
        try:
            check_key_set(k, iv, cv, is_, cs, hq, np.arange(n), granularity=gran)
        except AssertionError as e:
            raise AssertionError("case %d: heads %d/%d n %d per_q %s g %s: %s" % (case, hq, hk, n, per_q, gran, e))
