"""Thin ctypes binding of the C ABI in ``include/vsprefill.h``: same names, argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch serves as the device allocator and stream provider);
every step of the path runs inside the library's kernels.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libvsprefill.so")
_lib = None

EXPORTS = [
    "vs_rope_apply", "vs_index_score_workspace", "vs_index_score", "vs_select_budget_workspace", "vs_select_budget",
    "vs_sparse_prefill_workspace", "vs_sparse_prefill", "vs_sparse_prefill_tiled", "vs_sparse_prefill_chunk",
    "vs_sparse_prefill_static", "vs_dense_prefill", "vs_dense_prefill_chunk", "vs_validate_lists",
    "vs_sparse_prefill_tiles", "vs_sparse_prefill_counters", "vs_aggregate_workspace", "vs_aggregate",
    "vs_index_train_workspace", "vs_index_train_step",
    "vs_strerror", "vs_last_hip_error", "vs_version",
]


class VsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _load().vs_strerror(code).decode()
        if code == -5:
            msg += " hipError=%d" % _load().vs_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, code))


class _Indexer(ctypes.Structure):
    _fields_ = [("W_U", ctypes.c_void_p), ("b_U", ctypes.c_void_p), ("W_V", ctypes.c_void_p), ("W_S", ctypes.c_void_p),
                ("b_V", ctypes.c_float), ("b_S", ctypes.c_float), ("d_h", ctypes.c_int), ("act", ctypes.c_int)]


class _Budget(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("tau_v", ctypes.c_double), ("tau_s", ctypes.c_double),
                ("k_v", ctypes.c_int), ("k_s", ctypes.c_int), ("n_sink", ctypes.c_int), ("n_local", ctypes.c_int),
                ("cap_v", ctypes.c_int), ("cap_s", ctypes.c_int)]


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libvsprefill.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32, f64, sz = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_double,
                                  ctypes.c_size_t)
    L.vs_rope_apply.argtypes = [vp, i32, i64, i64, f64, i32, vp]
    L.vs_index_score_workspace.argtypes = [i32, i64, i32]
    L.vs_index_score_workspace.restype = sz
    L.vs_index_score.argtypes = [vp, vp, i32, i64, ctypes.POINTER(_Indexer), vp, vp, vp, sz, vp]
    L.vs_select_budget_workspace.argtypes = [i32, i64]
    L.vs_select_budget_workspace.restype = sz
    L.vs_select_budget.argtypes = [vp, vp, i32, i64, ctypes.POINTER(_Budget), vp, vp, vp, vp, vp, vp, sz, vp]
    L.vs_sparse_prefill_workspace.argtypes = [i32, i32, i32, i64]
    L.vs_sparse_prefill_workspace.restype = sz
    L.vs_sparse_prefill.argtypes = [vp, vp, vp, i32, i32, i64, f32, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    L.vs_sparse_prefill_tiled.argtypes = [vp, vp, vp, i32, i32, i64, f32, vp, vp, i32, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.vs_sparse_prefill_static.argtypes = [vp, vp, vp, i32, i32, i64, f32, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp]
    L.vs_dense_prefill.argtypes = [vp, vp, vp, i32, i32, i64, f32, vp, vp, vp]
    L.vs_sparse_prefill_chunk.argtypes = [vp, vp, vp, i32, i32, i64, i64, i64, f32, vp, vp, i32, vp, vp, i32, i32, i32, vp, vp,
                                          vp, sz, vp]
    L.vs_dense_prefill_chunk.argtypes = [vp, vp, vp, i32, i32, i64, i64, i64, f32, vp, vp, vp]
    L.vs_validate_lists.argtypes = [vp, vp, i32, i32, i64, vp, vp]
    L.vs_sparse_prefill_tiles.argtypes = [vp, sz, vp, ctypes.POINTER(ctypes.c_int64)]
    L.vs_sparse_prefill_counters.argtypes = [vp, sz, vp, ctypes.POINTER(ctypes.c_int64)]
    L.vs_aggregate_workspace.argtypes = [i32, i32, i32, i64]
    L.vs_aggregate_workspace.restype = sz
    L.vs_aggregate.argtypes = [vp, vp, i32, i32, i64, f32, vp, i32, vp, vp, vp, vp, i32, vp, vp, i32, i32, vp, vp, sz, vp]
    L.vs_index_train_workspace.argtypes = [i32, i64, i32]
    L.vs_index_train_workspace.restype = sz
    L.vs_index_train_step.argtypes = [vp, vp, i32, i64, ctypes.POINTER(_Indexer), vp, vp, f32, vp, vp, vp, vp, vp, vp, sz, vp]
    L.vs_strerror.argtypes = [i32]
    L.vs_strerror.restype = ctypes.c_char_p
    L.vs_last_hip_error.restype = i32
    L.vs_version.restype = ctypes.c_char_p
    for name in EXPORTS:
        getattr(L, name)
    _lib = L
    return L


def exported_symbols():
    """Names from include/vsprefill.h that the loaded library exports."""
    L = _load()
    return [n for n in EXPORTS if hasattr(L, n)]


def version():
    return _load().vs_version().decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc, where):
    if rc != 0:
        raise VsError(rc, where)


def _dev(t, dtype, what):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (what, dtype))
    return t


class IndexerWeights:
    """Device-resident VSIndexer parameters (one set per layer)."""

    def __init__(self, W_U, b_U, W_V, W_S, b_V=0.0, b_S=0.0, act=1):
        import torch
        self.W_U = _dev(W_U, torch.float32, "W_U")
        self.b_U = _dev(b_U, torch.float32, "b_U")
        self.W_V = _dev(W_V, torch.float32, "W_V")
        self.W_S = _dev(W_S, torch.float32, "W_S")
        self.d_h = int(W_U.shape[1])
        assert W_U.shape[0] == 256 and b_U.numel() == self.d_h and W_V.numel() == self.d_h and W_S.numel() == self.d_h
        self.b_V, self.b_S, self.act = float(b_V), float(b_S), int(act)

    def c_struct(self):
        return _Indexer(self.W_U.data_ptr(), self.b_U.data_ptr(), self.W_V.data_ptr(), self.W_S.data_ptr(),
                        self.b_V, self.b_S, self.d_h, self.act)


class Budget:
    def __init__(self, mode=0, tau_v=0.9, tau_s=0.9, k_v=0, k_s=0, n_sink=0, n_local=1, cap_v=0, cap_s=0):
        self.mode, self.tau_v, self.tau_s, self.k_v, self.k_s = mode, tau_v, tau_s, k_v, k_s
        self.n_sink, self.n_local, self.cap_v, self.cap_s = n_sink, n_local, cap_v, cap_s

    def c_struct(self):
        return _Budget(self.mode, self.tau_v, self.tau_s, self.k_v, self.k_s, self.n_sink, self.n_local,
                       self.cap_v, self.cap_s)


def rope_apply(x, pos0=0, theta_base=1e6, pairing=0, stream=None):
    import torch
    _dev(x, torch.bfloat16, "x")
    heads, n, d = x.shape
    assert d == 128
    _check(_load().vs_rope_apply(_ptr(x), heads, n, pos0, theta_base, pairing, _stream(stream)), "vs_rope_apply")
    return x


def index_score_workspace(kv_heads, n, d_h):
    return _load().vs_index_score_workspace(kv_heads, n, d_h)


def index_score(k, v, weights, a_v, a_s, ws, stream=None):
    import torch
    _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v")
    _dev(a_v, torch.float32, "a_v"); _dev(a_s, torch.float32, "a_s")
    kv_heads, n, d = k.shape
    assert d == 128 and v.shape == k.shape and a_v.shape == (kv_heads, n) and a_s.shape == (kv_heads, n)
    w = weights.c_struct()
    _check(_load().vs_index_score(_ptr(k), _ptr(v), kv_heads, n, ctypes.byref(w), _ptr(a_v), _ptr(a_s),
                                  _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "vs_index_score")
    return a_v, a_s


def select_budget_workspace(heads, n):
    return _load().vs_select_budget_workspace(heads, n)


def select_budget(a_v, a_s, budget, idx_v, cnt_v, idx_s, cnt_s, status, ws, stream=None):
    import torch
    _dev(a_v, torch.float32, "a_v"); _dev(a_s, torch.float32, "a_s")
    _dev(idx_v, torch.int32, "idx_v"); _dev(idx_s, torch.int32, "idx_s")
    _dev(cnt_v, torch.int32, "cnt_v"); _dev(cnt_s, torch.int32, "cnt_s")
    heads, n = a_v.shape
    assert a_s.shape == (heads, n) and idx_v.shape == (heads, budget.cap_v) and idx_s.shape == (heads, budget.cap_s)
    b = budget.c_struct()
    _check(_load().vs_select_budget(_ptr(a_v), _ptr(a_s), heads, n, ctypes.byref(b), _ptr(idx_v), _ptr(cnt_v),
                                    _ptr(idx_s), _ptr(cnt_s), _ptr(status), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "vs_select_budget")


def sparse_prefill_workspace(q_heads, kv_heads, index_heads, n):
    return _load().vs_sparse_prefill_workspace(q_heads, kv_heads, index_heads, n)


def sparse_prefill(q, k, v, idx_v, cnt_v, idx_s, cnt_s, o, lse, ws, scale=None, stream=None, slash_granularity=None,
                   pos0=None):
    """pos0 given: q / o hold a chunk of n_q rows at positions pos0 .. pos0 + n_q - 1, k / v all n_kv keys
    (vs_sparse_prefill_chunk)."""
    import torch
    if pos0 is not None:
        return _sparse_prefill_chunk(q, k, v, idx_v, cnt_v, idx_s, cnt_s, o, lse, ws, scale, stream, slash_granularity or 1, pos0)
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v"); _dev(o, torch.bfloat16, "o")
    _dev(idx_v, torch.int32, "idx_v"); _dev(idx_s, torch.int32, "idx_s")
    _dev(cnt_v, torch.int32, "cnt_v"); _dev(cnt_s, torch.int32, "cnt_s")
    q_heads, n, d = q.shape
    kv_heads = k.shape[0]
    assert d == 128 and k.shape == (kv_heads, n, 128) and v.shape == k.shape and o.shape == q.shape
    index_heads = idx_v.shape[0]
    assert idx_s.shape[0] == index_heads and cnt_v.numel() == index_heads and cnt_s.numel() == index_heads
    if lse is not None:
        _dev(lse, torch.float32, "lse")
        assert lse.shape == (q_heads, n)
    scale = 128 ** -0.5 if scale is None else scale
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    if slash_granularity is None:
        _check(_load().vs_sparse_prefill(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n, scale, _ptr(idx_v), _ptr(cnt_v),
                                         idx_v.shape[1], _ptr(idx_s), _ptr(cnt_s), idx_s.shape[1], index_heads,
                                         _ptr(o), _ptr(lse), _ptr(ws), ws_bytes, _stream(stream)), "vs_sparse_prefill")
    else:
        _check(_load().vs_sparse_prefill_tiled(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n, scale, _ptr(idx_v),
                                               _ptr(cnt_v), idx_v.shape[1], _ptr(idx_s), _ptr(cnt_s), idx_s.shape[1],
                                               index_heads, int(slash_granularity), _ptr(o), _ptr(lse), _ptr(ws), ws_bytes,
                                               _stream(stream)), "vs_sparse_prefill_tiled")
    return o


def _sparse_prefill_chunk(q, k, v, idx_v, cnt_v, idx_s, cnt_s, o, lse, ws, scale, stream, gran, pos0):
    import torch
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v"); _dev(o, torch.bfloat16, "o")
    _dev(idx_v, torch.int32, "idx_v"); _dev(idx_s, torch.int32, "idx_s")
    _dev(cnt_v, torch.int32, "cnt_v"); _dev(cnt_s, torch.int32, "cnt_s")
    q_heads, n_q, d = q.shape
    kv_heads, n_kv = k.shape[0], k.shape[1]
    assert d == 128 and k.shape == (kv_heads, n_kv, 128) and v.shape == k.shape and o.shape == q.shape
    index_heads = idx_v.shape[0]
    assert idx_s.shape[0] == index_heads and cnt_v.numel() == index_heads and cnt_s.numel() == index_heads
    if lse is not None:
        _dev(lse, torch.float32, "lse")
        assert lse.shape == (q_heads, n_q)
    scale = 128 ** -0.5 if scale is None else scale
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(_load().vs_sparse_prefill_chunk(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n_q, n_kv, int(pos0), scale,
                                           _ptr(idx_v), _ptr(cnt_v), idx_v.shape[1], _ptr(idx_s), _ptr(cnt_s),
                                           idx_s.shape[1], index_heads, int(gran), _ptr(o), _ptr(lse), _ptr(ws), ws_bytes,
                                           _stream(stream)), "vs_sparse_prefill_chunk")
    return o


def validate_lists(idx, cnt, n, report, stream=None):
    """report [heads] int32 (device): 0 or a bit-or of 1 (bad count), 2 (entry out of range), 4 (not strictly ascending)."""
    import torch
    _dev(idx, torch.int32, "idx"); _dev(cnt, torch.int32, "cnt"); _dev(report, torch.int32, "report")
    heads, cap = idx.shape
    assert cnt.numel() == heads and report.numel() == heads
    _check(_load().vs_validate_lists(_ptr(idx), _ptr(cnt), cap, heads, n, _ptr(report), _stream(stream)), "vs_validate_lists")
    return report


def sparse_prefill_static(q, k, v, idx_v, cnt_v, idx_s, cnt_s, o, lse, scale=None, stream=None):
    """vs_sparse_prefill without a workspace argument (the library's fixed per-GPU scratch array); allocates nothing."""
    import torch
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v"); _dev(o, torch.bfloat16, "o")
    _dev(idx_v, torch.int32, "idx_v"); _dev(idx_s, torch.int32, "idx_s")
    _dev(cnt_v, torch.int32, "cnt_v"); _dev(cnt_s, torch.int32, "cnt_s")
    q_heads, n, d = q.shape
    kv_heads = k.shape[0]
    assert d == 128 and k.shape == (kv_heads, n, 128) and v.shape == k.shape and o.shape == q.shape
    index_heads = idx_v.shape[0]
    assert idx_s.shape[0] == index_heads and cnt_v.numel() == index_heads and cnt_s.numel() == index_heads
    if lse is not None:
        _dev(lse, torch.float32, "lse")
        assert lse.shape == (q_heads, n)
    scale = 128 ** -0.5 if scale is None else scale
    _check(_load().vs_sparse_prefill_static(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n, scale, _ptr(idx_v),
                                            _ptr(cnt_v), idx_v.shape[1], _ptr(idx_s), _ptr(cnt_s), idx_s.shape[1],
                                            index_heads, _ptr(o), _ptr(lse), _stream(stream)), "vs_sparse_prefill_static")
    return o


def sparse_prefill_tiles(ws, stream=None):
    out = ctypes.c_int64(0)
    _check(_load().vs_sparse_prefill_tiles(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream), ctypes.byref(out)),
           "vs_sparse_prefill_tiles")
    return out.value


def sparse_prefill_counters(ws, stream=None):
    """(executed MFMA tiles, staged gather tiles, staged block tiles) of the last sparse call on this workspace."""
    out = (ctypes.c_int64 * 3)()
    _check(_load().vs_sparse_prefill_counters(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream), out),
           "vs_sparse_prefill_counters")
    return int(out[0]), int(out[1]), int(out[2])


def aggregate_workspace(q_heads, kv_heads, index_heads, n):
    return _load().vs_aggregate_workspace(q_heads, kv_heads, index_heads, n)


def aggregate(q, k, a_v, a_s, ws, lse=None, lists=None, recall=None, scale=None, stream=None):
    """a_v, a_s: [out_heads, n] fp32 with out_heads = q_heads or kv_heads.  lists = (idx_v, cnt_v, idx_s, cnt_s) and
    recall [out_heads] fp32 go together."""
    import torch
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(a_v, torch.float32, "a_v"); _dev(a_s, torch.float32, "a_s")
    q_heads, n, d = q.shape
    kv_heads = k.shape[0]
    out_heads = a_v.shape[0]
    assert d == 128 and k.shape == (kv_heads, n, 128) and a_v.shape == (out_heads, n) and a_s.shape == a_v.shape
    if lse is not None:
        _dev(lse, torch.float32, "lse")
        assert lse.shape == (q_heads, n)
    idx_v = cnt_v = idx_s = cnt_s = None
    cap_v = cap_s = index_heads = 0
    if recall is not None:
        _dev(recall, torch.float32, "recall")
        assert recall.numel() == out_heads and lists is not None
        idx_v, cnt_v, idx_s, cnt_s = lists
        _dev(idx_v, torch.int32, "idx_v"); _dev(idx_s, torch.int32, "idx_s")
        _dev(cnt_v, torch.int32, "cnt_v"); _dev(cnt_s, torch.int32, "cnt_s")
        index_heads = idx_v.shape[0]
        assert idx_s.shape[0] == index_heads and cnt_v.numel() == index_heads and cnt_s.numel() == index_heads
        cap_v, cap_s = idx_v.shape[1], idx_s.shape[1]
    scale = 128 ** -0.5 if scale is None else scale
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(_load().vs_aggregate(_ptr(q), _ptr(k), q_heads, kv_heads, n, scale, _ptr(lse), out_heads, _ptr(a_v), _ptr(a_s),
                                _ptr(idx_v), _ptr(cnt_v), cap_v, _ptr(idx_s), _ptr(cnt_s), cap_s, index_heads,
                                _ptr(recall), _ptr(ws), ws_bytes, _stream(stream)), "vs_aggregate")
    return a_v, a_s


def index_train_workspace(kv_heads, n, d_h):
    return _load().vs_index_train_workspace(kv_heads, n, d_h)


def index_train_step(k, v, weights, t_v, t_s, loss, dW_U, db_U, dW_V, dW_S, ws, eps=1e-30, stream=None):
    """Loss KL(A^_v || t_v) + KL(A^_s || t_s) (mean over KV heads) and its gradient with respect to the indexer parameters."""
    import torch
    _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v")
    _dev(t_v, torch.float32, "t_v"); _dev(t_s, torch.float32, "t_s"); _dev(loss, torch.float32, "loss")
    for name, t in (("dW_U", dW_U), ("db_U", db_U), ("dW_V", dW_V), ("dW_S", dW_S)):
        _dev(t, torch.float32, name)
    kv_heads, n, d = k.shape
    d_h = weights.d_h
    assert d == 128 and v.shape == k.shape and t_v.shape == (kv_heads, n) and t_s.shape == (kv_heads, n)
    assert dW_U.shape == (256, d_h) and db_U.numel() == d_h and dW_V.numel() == d_h and dW_S.numel() == d_h and loss.numel() == 1
    w = weights.c_struct()
    _check(_load().vs_index_train_step(_ptr(k), _ptr(v), kv_heads, n, ctypes.byref(w), _ptr(t_v), _ptr(t_s), eps, _ptr(loss),
                                       _ptr(dW_U), _ptr(db_U), _ptr(dW_V), _ptr(dW_S), _ptr(ws),
                                       0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "vs_index_train_step")
    return loss


def dense_prefill(q, k, v, o, lse=None, scale=None, stream=None, pos0=None):
    """pos0 given: q / o hold a chunk of n_q rows at positions pos0 .. pos0 + n_q - 1 (vs_dense_prefill_chunk)."""
    import torch
    _dev(q, torch.bfloat16, "q"); _dev(k, torch.bfloat16, "k"); _dev(v, torch.bfloat16, "v"); _dev(o, torch.bfloat16, "o")
    q_heads, n_q, d = q.shape
    kv_heads, n = k.shape[0], k.shape[1]
    assert d == 128 and k.shape == (kv_heads, n, 128) and v.shape == k.shape and o.shape == q.shape
    assert pos0 is not None or n_q == n
    if lse is not None:
        _dev(lse, torch.float32, "lse")
        assert lse.shape == (q_heads, n_q)
    scale = 128 ** -0.5 if scale is None else scale
    if pos0 is None:
        _check(_load().vs_dense_prefill(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n, scale, _ptr(o), _ptr(lse),
                                        _stream(stream)), "vs_dense_prefill")
    else:
        _check(_load().vs_dense_prefill_chunk(_ptr(q), _ptr(k), _ptr(v), q_heads, kv_heads, n_q, n, int(pos0), scale, _ptr(o),
                                              _ptr(lse), _stream(stream)), "vs_dense_prefill_chunk")
    return o
