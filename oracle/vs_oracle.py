"""ctypes front-end of ``vs_oracle.cpp`` (fp64 definitions of the path; test infrastructure only).

bf16 tensors travel as ``numpy.uint16`` arrays holding the raw bit patterns.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vs_oracle.cpp")
_LIB = os.path.join(_HERE, "libvs_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with g++ (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC",
                               "-pthread", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.vso_f64_to_bf16.restype = ctypes.c_uint16
        L.vso_f64_to_bf16.argtypes = [ctypes.c_double]
        L.vso_bf16_to_f64.restype = ctypes.c_double
        L.vso_bf16_to_f64.argtypes = [ctypes.c_uint16]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def f64_to_bf16(x):
    L = _load()
    x = np.asarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    xf, of = x.reshape(-1), out.reshape(-1)
    for i in range(xf.size):
        of[i] = L.vso_f64_to_bf16(float(xf[i]))
    return out


def bf16_to_f64(b):
    b = np.asarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rope_f64(x, pos0=0, theta_base=1e4, pairing=0):
    """x: [heads, n, d] float64 -> rotated copy."""
    L = _load()
    x = np.array(x, dtype=np.float64, order="C", copy=True)
    h, n, d = x.shape
    rc = L.vso_rope_f64(_p(x), ctypes.c_int(h), ctypes.c_int64(n), ctypes.c_int(d), ctypes.c_int64(pos0),
                        ctypes.c_double(theta_base), ctypes.c_int(pairing))
    assert rc == 0, rc
    return x


def rope_bf16(x, pos0=0, theta_base=1e4, pairing=0, threads=0):
    """x: [heads, n, d] uint16 (bf16 bits) -> rotated copy, rounded once to bf16."""
    L = _load()
    x = np.array(x, dtype=np.uint16, order="C", copy=True)
    h, n, d = x.shape
    rc = L.vso_rope_bf16(_p(x), ctypes.c_int(h), ctypes.c_int64(n), ctypes.c_int(d), ctypes.c_int64(pos0),
                         ctypes.c_double(theta_base), ctypes.c_int(pairing), ctypes.c_int(threads))
    assert rc == 0, rc
    return x


def index_score(k, v, W_U, b_U, W_V, W_S, b_V=0.0, b_S=0.0, act=1, threads=0, return_logits=False):
    """k, v: [kv_heads, n, d] uint16; W_U: [2d, d_h] fp32.  Returns (a_v, a_s) float64 [kv_heads, n]."""
    L = _load()
    k = _c(k, np.uint16); v = _c(v, np.uint16)
    W_U = _c(W_U, np.float32); b_U = _c(b_U, np.float32); W_V = _c(W_V, np.float32); W_S = _c(W_S, np.float32)
    hk, n, d = k.shape
    d_h = W_U.shape[1]
    assert W_U.shape[0] == 2 * d and b_U.shape == (d_h,) and W_V.shape == (d_h,) and W_S.shape == (d_h,)
    a_v = np.empty((hk, n), dtype=np.float64); a_s = np.empty((hk, n), dtype=np.float64)
    lv = np.empty((hk, n), dtype=np.float64) if return_logits else None
    ls = np.empty((hk, n), dtype=np.float64) if return_logits else None
    rc = L.vso_index_score(_p(k), _p(v), ctypes.c_int(hk), ctypes.c_int64(n), ctypes.c_int(d),
                           _p(W_U), _p(b_U), _p(W_V), _p(W_S), ctypes.c_float(b_V), ctypes.c_float(b_S),
                           ctypes.c_int(d_h), ctypes.c_int(act), _p(a_v), _p(a_s), _p(lv), _p(ls),
                           ctypes.c_int(threads))
    assert rc == 0, rc
    return (a_v, a_s, lv, ls) if return_logits else (a_v, a_s)


def select(scores, mode=0, tau=0.9, k_fixed=0, n_forced=0, cap=None):
    """scores: [heads, n] fp32.  Returns (idx [heads, cap] int32, cnt [heads], status [heads], k [heads])."""
    L = _load()
    scores = _c(scores, np.float32)
    heads, n = scores.shape
    cap = n if cap is None else cap
    idx = np.full((heads, cap), -1, dtype=np.int32)
    cnt = np.zeros(heads, dtype=np.int32); status = np.zeros(heads, dtype=np.int32)
    k = np.zeros(heads, dtype=np.int64)
    rc = L.vso_select(_p(scores), ctypes.c_int(heads), ctypes.c_int64(n), ctypes.c_int(mode), ctypes.c_double(tau),
                      ctypes.c_int64(k_fixed), ctypes.c_int64(n_forced), ctypes.c_int64(cap),
                      _p(idx), _p(cnt), _p(status), _p(k))
    if rc != 0:
        raise ValueError("vso_select rc=%d" % rc)
    return idx, cnt, status, k


def _lists(idx, cnt):
    idx = _c(idx, np.int32); cnt = _c(cnt, np.int32)
    assert idx.ndim == 2 and cnt.shape == (idx.shape[0],)
    return idx, cnt


def sparse_attention(q, k, v, idx_v, cnt_v, idx_s, cnt_s, scale=None, rows=None, threads=0, return_live=False,
                     granularity=1, pos0=0):
    """q: [Hq, n_q, d], k, v: [Hkv, n, d] uint16.  idx_*: [index_heads, cap] int32 ascending, cnt_*: [index_heads].
    The query rows are the positions pos0 .. pos0 + n_q - 1 (chunked prefill; pos0 + n_q <= n); `rows` are local row
    numbers.  granularity g > 1: tile-granular slash variant (a key is kept for a position if any position of its aligned
    g-block reaches it through a selected offset).
    Returns (out [Hq, n_rows, d] f64, lse [Hq, n_rows] f64[, live [Hq, n_rows] int64])."""
    L = _load()
    q = _c(q, np.uint16); k = _c(k, np.uint16); v = _c(v, np.uint16)
    hq, n_q, d = q.shape
    hk, n = k.shape[0], k.shape[1]
    idx_v, cnt_v = _lists(idx_v, cnt_v); idx_s, cnt_s = _lists(idx_s, cnt_s)
    ih = idx_v.shape[0]
    assert idx_s.shape[0] == ih
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    rows_a = None if rows is None else _c(rows, np.int64)
    nr = n_q if rows is None else rows_a.size
    out = np.empty((hq, nr, d), dtype=np.float64); lse = np.empty((hq, nr), dtype=np.float64)
    live = np.empty((hq, nr), dtype=np.int64)
    rc = L.vso_sparse_attention(_p(q), _p(k), _p(v), ctypes.c_int(hq), ctypes.c_int(hk), ctypes.c_int64(n),
                                ctypes.c_int(d), ctypes.c_double(scale),
                                _p(idx_v), _p(cnt_v), ctypes.c_int64(idx_v.shape[1]),
                                _p(idx_s), _p(cnt_s), ctypes.c_int64(idx_s.shape[1]), ctypes.c_int(ih),
                                ctypes.c_int64(granularity), _p(rows_a), ctypes.c_int64(nr), ctypes.c_int64(n_q),
                                ctypes.c_int64(pos0), _p(out), _p(lse), _p(live), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("vso_sparse_attention rc=%d" % rc)
    return (out, lse, live) if return_live else (out, lse)


def dense_attention(q, k, v, scale=None, rows=None, threads=0, pos0=0):
    L = _load()
    q = _c(q, np.uint16); k = _c(k, np.uint16); v = _c(v, np.uint16)
    hq, n_q, d = q.shape
    hk, n = k.shape[0], k.shape[1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    rows_a = None if rows is None else _c(rows, np.int64)
    nr = n_q if rows is None else rows_a.size
    out = np.empty((hq, nr, d), dtype=np.float64); lse = np.empty((hq, nr), dtype=np.float64)
    rc = L.vso_dense_attention(_p(q), _p(k), _p(v), ctypes.c_int(hq), ctypes.c_int(hk), ctypes.c_int64(n),
                               ctypes.c_int(d), ctypes.c_double(scale), _p(rows_a), ctypes.c_int64(nr),
                               ctypes.c_int64(n_q), ctypes.c_int64(pos0), _p(out), _p(lse), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("vso_dense_attention rc=%d" % rc)
    return out, lse


def vs_aggregate(q, k, scale=None, idx_v=None, idx_s=None):
    """One head: q, k [n, d] uint16.  Returns (A_v, A_s) (each sums to 1) and, when lists are given, the recall."""
    L = _load()
    q = _c(q, np.uint16); k = _c(k, np.uint16)
    n, d = q.shape
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    a_v = np.empty(n, dtype=np.float64); a_s = np.empty(n, dtype=np.float64)
    want = idx_v is not None or idx_s is not None
    iv = _c(idx_v if idx_v is not None else [], np.int32); is_ = _c(idx_s if idx_s is not None else [], np.int32)
    rec = ctypes.c_double(0.0)
    rc = L.vso_vs_aggregate(_p(q), _p(k), ctypes.c_int64(n), ctypes.c_int(d), ctypes.c_double(scale), _p(a_v), _p(a_s),
                            _p(iv), ctypes.c_int64(iv.size), _p(is_), ctypes.c_int64(is_.size),
                            ctypes.byref(rec) if want else None)
    assert rc == 0, rc
    return (a_v, a_s, rec.value) if want else (a_v, a_s)


TRAIN_EPS = 1e-30


def index_train(k, v, W_U, b_U, W_V, W_S, t_v, t_s, b_V=0.0, b_S=0.0, act=1, eps=TRAIN_EPS, return_glogits=False):
    """Distillation loss L = mean over heads of KL(A^_v || A_v) + KL(A^_s || A_s) and its gradient.
    k, v: [kv_heads, n, d] uint16; targets t_v, t_s: [kv_heads, n].  Returns (loss, dW_U, db_U, dW_V, dW_S) in float64
    (and the gradients with respect to the logits when asked)."""
    L = _load()
    k = _c(k, np.uint16); v = _c(v, np.uint16)
    W_U = _c(W_U, np.float32); b_U = _c(b_U, np.float32); W_V = _c(W_V, np.float32); W_S = _c(W_S, np.float32)
    t_v = _c(t_v, np.float64); t_s = _c(t_s, np.float64)
    hk, n, d = k.shape
    d_h = W_U.shape[1]
    assert W_U.shape[0] == 2 * d and t_v.shape == (hk, n) and t_s.shape == (hk, n)
    loss = ctypes.c_double(0.0)
    dW_U = np.empty((2 * d, d_h)); db_U = np.empty(d_h); dW_V = np.empty(d_h); dW_S = np.empty(d_h)
    g_v = np.empty((hk, n)) if return_glogits else None
    g_s = np.empty((hk, n)) if return_glogits else None
    rc = L.vso_index_train(_p(k), _p(v), ctypes.c_int(hk), ctypes.c_int64(n), ctypes.c_int(d), _p(W_U), _p(b_U), _p(W_V),
                           _p(W_S), ctypes.c_float(b_V), ctypes.c_float(b_S), ctypes.c_int(d_h), ctypes.c_int(act),
                           _p(t_v), _p(t_s), ctypes.c_double(eps), ctypes.byref(loss), _p(dW_U), _p(db_U), _p(dW_V), _p(dW_S),
                           _p(g_v), _p(g_s))
    assert rc == 0, rc
    out = (loss.value, dW_U, db_U, dW_V, dW_S)
    return out + (g_v, g_s) if return_glogits else out
