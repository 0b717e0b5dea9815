"""Pins for the VSIndexer oracle (Sec. "VSIndexer Design")."""
import numpy as np
import pytest
import torch

import oracle
from brute import bits_to_f64, f32_to_bf16_bits


def make(rng, hk, n, d, d_h):
    k = f32_to_bf16_bits(rng.standard_normal((hk, n, d)).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((hk, n, d)).astype(np.float32))
    W_U = (rng.uniform(-1, 1, (2 * d, d_h)) / np.sqrt(2 * d)).astype(np.float32)
    b_U = (rng.uniform(-1, 1, d_h) / np.sqrt(2 * d)).astype(np.float32)
    W_V = rng.uniform(-1, 1, d_h).astype(np.float32)
    W_S = rng.uniform(-1, 1, d_h).astype(np.float32)
    return k, v, W_U, b_U, W_V, W_S


@pytest.mark.parametrize("act", [0, 1])
def test_against_library_layers(act):
    """The same network assembled from torch's fp64 linear / silu / gelu(erf) / softmax routines."""
    rng = np.random.default_rng(act)
    hk, n, d, d_h = 2, 50, 16, 24
    k, v, W_U, b_U, W_V, W_S = make(rng, hk, n, d, d_h)
    a_v, a_s, lv, ls = oracle.index_score(k, v, W_U, b_U, W_V, W_S, 0.3, -0.2, act=act, return_logits=True)
    X = torch.cat([torch.from_numpy(bits_to_f64(k)), torch.from_numpy(bits_to_f64(v))], dim=-1)
    Z = torch.nn.functional.linear(X, torch.from_numpy(W_U.astype(np.float64)).T, torch.from_numpy(b_U.astype(np.float64)))
    Z = torch.nn.functional.silu(Z) if act == 0 else torch.nn.functional.gelu(Z, approximate="none")
    lv_ref = Z @ torch.from_numpy(W_V.astype(np.float64)) + np.float64(np.float32(0.3))
    ls_ref = Z @ torch.from_numpy(W_S.astype(np.float64)) + np.float64(np.float32(-0.2))
    np.testing.assert_allclose(lv, lv_ref.numpy(), atol=1e-12)
    np.testing.assert_allclose(ls, ls_ref.numpy(), atol=1e-12)
    np.testing.assert_allclose(a_v, torch.softmax(lv_ref, dim=-1).numpy(), atol=1e-14)
    np.testing.assert_allclose(a_s, torch.softmax(ls_ref, dim=-1).numpy(), atol=1e-14)


def test_hand_computable_single_unit():
    """d = 2, d_h = 1, W_U picks k_0 only for the vertical path: logits are silu(k_0) * w."""
    k = f32_to_bf16_bits(np.array([[[1.0, 5.0], [-2.0, 7.0], [0.5, -3.0]]], dtype=np.float32))
    v = f32_to_bf16_bits(np.array([[[9.0, 9.0], [8.0, 8.0], [7.0, 7.0]]], dtype=np.float32))
    W_U = np.array([[1.0], [0.0], [0.0], [0.0]], dtype=np.float32)
    a_v, a_s = oracle.index_score(k, v, W_U, np.zeros(1, np.float32), np.array([2.0], np.float32),
                                  np.array([-1.0], np.float32), act=0)
    x = np.array([1.0, -2.0, 0.5])
    z = x / (1 + np.exp(-x))
    for a, w in ((a_v, 2.0), (a_s, -1.0)):
        e = np.exp(w * z)
        np.testing.assert_allclose(a[0], e / e.sum(), atol=1e-15)
    # the value half of X is wired to rows d..2d-1 of W_U
    W_U2 = np.array([[0.0], [0.0], [0.0], [1.0]], dtype=np.float32)
    a_v2, _ = oracle.index_score(k, v, W_U2, np.zeros(1, np.float32), np.array([1.0], np.float32),
                                 np.array([0.0], np.float32), act=1)
    from math import erf, sqrt
    x = np.array([9.0, 8.0, 7.0])
    z = np.array([0.5 * t * (1 + erf(t / sqrt(2))) for t in x])
    np.testing.assert_allclose(a_v2[0], np.exp(z) / np.exp(z).sum(), atol=1e-15)


def test_structural_properties():
    rng = np.random.default_rng(4)
    hk, n, d, d_h = 2, 64, 8, 16
    k, v, W_U, b_U, W_V, W_S = make(rng, hk, n, d, d_h)
    a_v, a_s = oracle.index_score(k, v, W_U, b_U, W_V, W_S)
    np.testing.assert_allclose(a_v.sum(axis=1), 1.0, atol=1e-14)
    np.testing.assert_allclose(a_s.sum(axis=1), 1.0, atol=1e-14)
    # output biases cancel inside the softmax over positions
    b_v, b_s = oracle.index_score(k, v, W_U, b_U, W_V, W_S, b_V=3.5, b_S=-7.25)
    np.testing.assert_allclose(a_v, b_v, atol=1e-15)
    np.testing.assert_allclose(a_s, b_s, atol=1e-15)
    # zero down-projection => uniform scores
    u_v, u_s = oracle.index_score(k, v, W_U, b_U, np.zeros_like(W_V), W_S)
    np.testing.assert_allclose(u_v, 1.0 / n, atol=1e-16)
    np.testing.assert_allclose(u_s, a_s, atol=1e-15)
    # no positional dependence inside the net: permuting tokens permutes the scores
    perm = rng.permutation(n)
    p_v, p_s = oracle.index_score(k[:, perm], v[:, perm], W_U, b_U, W_V, W_S)
    np.testing.assert_allclose(p_v, a_v[:, perm], atol=1e-15)
    np.testing.assert_allclose(p_s, a_s[:, perm], atol=1e-15)
    # heads are independent and share the weights
    h_v, _ = oracle.index_score(k[1:], v[1:], W_U, b_U, W_V, W_S)
    np.testing.assert_array_equal(h_v[0], a_v[1])
