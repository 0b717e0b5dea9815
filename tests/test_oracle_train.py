"""Pins for the distillation-step oracle (CPU only): loss KL(A^_v || A_v) + KL(A^_s || A_s) of paragraph "Loss
function design" and its gradient with respect to the indexer parameters.  Pinned by torch autograd in fp64 on the same
network assembled from library ops, by central finite differences of the loss, by the closed form of the gradient with
respect to the logits, and by special cases (target == prediction, bias invariance)."""
import numpy as np
import pytest
import torch

import oracle
from brute import bits_to_f64, f32_to_bf16_bits


def _setup(seed, hk=2, n=19, d=4, d_h=6):
    rng = np.random.default_rng(seed)
    k = f32_to_bf16_bits(rng.standard_normal((hk, n, d)).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((hk, n, d)).astype(np.float32))
    W_U = rng.uniform(-0.7, 0.7, (2 * d, d_h)).astype(np.float32)
    b_U = rng.uniform(-0.5, 0.5, d_h).astype(np.float32)
    W_V = rng.uniform(-2, 2, d_h).astype(np.float32)
    W_S = rng.uniform(-2, 2, d_h).astype(np.float32)
    t = rng.standard_normal((2, hk, n))
    t = np.exp(t) / np.exp(t).sum(axis=2, keepdims=True)
    return k, v, (W_U, b_U, W_V, W_S), t[0], t[1]


def _torch_loss(k, v, W, t_v, t_s, act, b_V=0.0, b_S=0.0):
    """The same network and loss assembled from torch fp64 library ops (no oracle code)."""
    x = torch.from_numpy(np.concatenate([bits_to_f64(k), bits_to_f64(v)], axis=2))            # [hk, n, 2d]
    W_U, b_U, W_V, W_S = [torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in W]
    pre = x @ W_U + b_U
    z = torch.nn.functional.silu(pre) if act == 0 else torch.nn.functional.gelu(pre)          # erf form
    loss = 0.0
    for w, b, t in ((W_V, b_V, t_v), (W_S, b_S, t_s)):
        logp = torch.log_softmax(z @ w + b, dim=1)
        # F.kl_div(input = log Q, target = P) is sum P (log P - input): KL(P || Q); the paper's KL(A^ || A) has P = A^
        loss = loss + torch.nn.functional.kl_div(torch.log(torch.from_numpy(t)), logp, reduction="sum", log_target=True)
    loss = loss / x.shape[0]
    loss.backward()
    return loss.item(), [p.grad.numpy() for p in (W_U, b_U, W_V, W_S)]


@pytest.mark.parametrize("act", [0, 1])
def test_matches_torch_autograd_fp64(act):
    k, v, W, t_v, t_s = _setup(10 + act)
    loss, dW_U, db_U, dW_V, dW_S = oracle.index_train(k, v, *W, t_v, t_s, 0.3, -0.2, act=act)
    ref_loss, ref = _torch_loss(k, v, W, t_v, t_s, act, 0.3, -0.2)
    np.testing.assert_allclose(loss, ref_loss, rtol=1e-12)
    for got, want in zip((dW_U, db_U, dW_V, dW_S), ref):
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-13)
    assert loss > 0


def test_central_finite_differences():
    """Perturb single parameters (fp32-representable steps) and difference the oracle's own loss."""
    k, v, W, t_v, t_s = _setup(3, hk=1, n=11, d=2, d_h=3)
    W = [np.round(a * 64) / 64 for a in W]                 # coarse values: the +-h copies stay exact in fp32
    W = [a.astype(np.float32) for a in W]
    _, dW_U, db_U, dW_V, dW_S = oracle.index_train(k, v, *W, t_v, t_s, act=1)
    h = 2.0 ** -10
    for which, grad in ((0, dW_U), (1, db_U), (2, dW_V), (3, dW_S)):
        it = np.ndindex(grad.shape)
        for idx in it:
            lo = [a.copy() for a in W]; hi = [a.copy() for a in W]
            lo[which][idx] -= h; hi[which][idx] += h
            fd = (oracle.index_train(k, v, *hi, t_v, t_s, act=1)[0] - oracle.index_train(k, v, *lo, t_v, t_s, act=1)[0]) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-5 * max(1.0, abs(grad[idx])), (which, idx, fd, grad[idx])


def test_logit_gradient_closed_form_and_special_cases():
    k, v, W, t_v, t_s = _setup(5)
    a_v, a_s = oracle.index_score(k, v, *W, act=1)
    loss, *_grads, g_v, g_s = oracle.index_train(k, v, *W, t_v, t_s, act=1, return_glogits=True)
    hk = k.shape[0]
    kl_v = (a_v * (np.log(a_v) - np.log(t_v))).sum(axis=1)
    kl_s = (a_s * (np.log(a_s) - np.log(t_s))).sum(axis=1)
    np.testing.assert_allclose(loss, (kl_v + kl_s).mean(), rtol=1e-12)
    np.testing.assert_allclose(g_v, a_v * (np.log(a_v) - np.log(t_v) - kl_v[:, None]) / hk, rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(g_s, a_s * (np.log(a_s) - np.log(t_s) - kl_s[:, None]) / hk, rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(g_v.sum(axis=1), 0.0, atol=1e-14)      # a shift of all logits changes nothing
    # target == prediction: zero loss, zero gradient
    loss0, dW_U, db_U, dW_V, dW_S = oracle.index_train(k, v, *W, a_v, a_s, act=1)
    assert abs(loss0) < 1e-13
    for g in (dW_U, db_U, dW_V, dW_S):
        assert np.abs(g).max() < 1e-12
    # the scalar output biases do not matter; a zero target entry is floored, not infinite
    l1 = oracle.index_train(k, v, *W, t_v, t_s, 5.0, -7.0, act=1)[0]
    np.testing.assert_allclose(l1, loss, rtol=1e-12)
    t0 = t_v.copy(); t0[0, 3] = 0.0
    l2 = oracle.index_train(k, v, *W, t0, t_s, act=1)[0]
    assert np.isfinite(l2) and l2 > loss
    np.testing.assert_allclose(l2 - loss, a_v[0, 3] * (np.log(t_v[0, 3]) - np.log(oracle.TRAIN_EPS)) / hk, rtol=1e-9)
