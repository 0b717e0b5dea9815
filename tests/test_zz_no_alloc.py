"""vs_sparse_prefill_static (the entry point that allocates nothing: its scratch is the library's fixed per-GPU array)
against vs_sparse_prefill on a caller workspace, through the C ABI: same kernels, so outputs must be identical bit for
bit, on two calls in a row that share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2603_04460_amd as vs
from gpu_util import make_qkv, lists

pytestmark = pytest.mark.gpu


def _case(seed, hq, hk, n, nv, ns):
    rng = np.random.default_rng(seed)
    (q, k, v), _ = make_qkv(seed, hq, hk, n)
    sv = [np.unique(np.concatenate([[0, 1], rng.choice(n, size=nv, replace=False)])) for _ in range(hk)]
    ss = [np.unique(np.concatenate([np.arange(min(40, n)), rng.choice(n, size=ns, replace=False)])) for _ in range(hk)]
    iv, cv = lists(sv)
    is_, cs = lists(ss)
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    return q, k, v, f(iv), f(cv), f(is_), f(cs)


def test_static_scratch_matches_workspace_entry_point():
    for seed, hq, hk, n, nv, ns in ((41, 8, 2, 5000, 700, 90), (42, 4, 1, 777, 60, 25)):   # large call, then a smaller one
        q, k, v, iv, cv, is_, cs = _case(seed, hq, hk, n, nv, ns)
        ws = torch.empty(vs.sparse_prefill_workspace(hq, hk, hk, n), dtype=torch.uint8, device="cuda")
        o_ref = torch.full_like(q, float("nan"))
        lse_ref = torch.full((hq, n), float("nan"), dtype=torch.float32, device="cuda")
        vs.sparse_prefill(q, k, v, iv, cv, is_, cs, o_ref, lse_ref, ws)
        o = torch.full_like(q, float("nan"))
        lse = torch.full((hq, n), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        # cumulative count of allocations made through torch: unlike the bytes in use, it cannot fall when the garbage
        # collector frees tensors of earlier tests during the call
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        vs.sparse_prefill_static(q, k, v, iv, cv, is_, cs, o, lse)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        assert torch.isfinite(o.float()).all()
        assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), "n = %d" % n
        assert torch.equal(lse, lse_ref), "n = %d" % n


def test_static_scratch_rejects_what_does_not_fit():
    hq, hk, n = 4, 4, 64
    (q, k, v), _ = make_qkv(5, hq, hk, n)
    z = torch.zeros((hk, 4), dtype=torch.int32, device="cuda")
    c = torch.ones(hk, dtype=torch.int32, device="cuda")
    o = torch.empty_like(q)
    vs.sparse_prefill_static(q, k, v, z, c, z, c, o, None)                 # tiny: fits
    # a size class that cannot fit the fixed array is refused on the host, before any launch (shapes only matter:
    # the check precedes every access), with its own error code
    import ctypes
    from paper_2603_04460_amd import binding
    L = binding._load()
    big_n, heads = 1 << 20, 32
    assert vs.sparse_prefill_workspace(heads, heads, heads, big_n) > 4 << 20
    p = ctypes.c_void_p(q.data_ptr())
    rc = L.vs_sparse_prefill_static(p, p, p, heads, heads, big_n, 0.0883883, ctypes.c_void_p(z.data_ptr()),
                                    ctypes.c_void_p(c.data_ptr()), 4, ctypes.c_void_p(z.data_ptr()),
                                    ctypes.c_void_p(c.data_ptr()), 4, heads, ctypes.c_void_p(o.data_ptr()), None, None)
    assert rc == -6
    assert b"scratch" in L.vs_strerror(rc)
    torch.cuda.synchronize()
