"""GPU parity of vs_index_train_step (distillation loss KL(A^_v || A_v) + KL(A^_s || A_s) and its gradient with respect
to the indexer parameters) against the fp64 oracle, through the C ABI.  Bar: 1e-3 relative on the loss; gradients 1e-3
relative to the largest entry of the tensor they belong to (entries that are themselves small come from cancellation
over thousands of tokens and carry no more digits than that) and 1e-3 element-wise on the entries that are not small."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_04460_amd as vs
import synth

pytestmark = pytest.mark.gpu


def _targets(rng, hk, n):
    t = rng.standard_normal((2, hk, n)) * 2.0
    t = np.exp(t - t.max(axis=2, keepdims=True))
    t = (t / t.sum(axis=2, keepdims=True)).astype(np.float32)
    return t[0], t[1]


def _gpu_step(k, v, W, act, t_v, t_s, eps=1e-30):
    hk, n, _ = k.shape
    d_h = W[0].shape[1]
    w = vs.IndexerWeights(*[torch.from_numpy(x).cuda() for x in W], 0.4, -0.3, act)
    ws = torch.empty(vs.index_train_workspace(hk, n, d_h), dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    g = [torch.full(s, float("nan"), dtype=torch.float32, device="cuda") for s in ((256, d_h), (d_h,), (d_h,), (d_h,))]
    vs.index_train_step(k, v, w, torch.from_numpy(t_v).cuda(), torch.from_numpy(t_s).cuda(), loss, *g, ws, eps=eps)
    torch.cuda.synchronize()
    return loss.item(), [x.cpu().numpy().astype(np.float64) for x in g]


def _check(got, ref, name):
    scale = np.abs(ref).max()
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), name
    assert err.max() <= 1e-3 * scale, "%s: error %.3g of scale %.3g" % (name, err.max(), scale)
    big = np.abs(ref) >= 0.05 * scale
    assert (err[big] <= 1e-3 * np.abs(ref[big])).all(), "%s: element-wise" % name


@pytest.mark.parametrize("hk,n,d_h,act", [(2, 1000, 256, 1), (1, 333, 64, 0), (3, 700, 128, 1), (2, 257, 1024, 0), (1, 31, 192, 1)])
def test_train_step_matches_oracle(hk, n, d_h, act):
    rng = np.random.default_rng(n + d_h)
    _, k, v = synth.qkv(70 + n, 1, hk, n, local_structure=True)
    W = synth.indexer_weights(n, d_h, act, gain=4.0)
    t_v, t_s = _targets(rng, hk, n)
    if n > 40:
        t_v[0, 17] = 0.0                                     # a zero target entry: floored by eps, finite everywhere
    loss, (dW_U, db_U, dW_V, dW_S) = _gpu_step(k.cuda(), v.cuda(), W, act, t_v, t_s)
    ref = oracle.index_train(synth.to_bits(k), synth.to_bits(v), *W, t_v.astype(np.float64), t_s.astype(np.float64), 0.4, -0.3,
                             act=act)
    assert abs(loss - ref[0]) <= 1e-3 * abs(ref[0]), (loss, ref[0])
    for got, want, name in zip((dW_U, db_U, dW_V, dW_S), ref[1:], ("dW_U", "db_U", "dW_V", "dW_S")):
        _check(got, want, name)


def test_train_step_on_aggregated_attention_targets_and_descent():
    """Targets from vs_aggregate (the distillation targets of the paper, here of synthetic Q / K); the step is
    deterministic, and a small move against the gradient lowers the loss."""
    hq, hk, n, d_h = 8, 2, 1536, 256
    q, k, v = synth.qkv(99, hq, hk, n, local_structure=True)
    q, k, v = q.cuda(), k.cuda(), v.cuda()
    vs.rope_apply(q, 0, 1e6)
    vs.rope_apply(k, 0, 1e6)
    t_v = torch.empty((hk, n), dtype=torch.float32, device="cuda"); t_s = torch.empty_like(t_v)
    wsa = torch.empty(vs.aggregate_workspace(hq, hk, 0, n), dtype=torch.uint8, device="cuda")
    vs.aggregate(q, k, t_v, t_s, wsa)
    torch.cuda.synchronize()
    W = synth.indexer_weights(99, d_h, 1, gain=4.0)
    tv, ts = t_v.cpu().numpy(), t_s.cpu().numpy()
    loss, grads = _gpu_step(k, v, W, 1, tv, ts)
    loss2, grads2 = _gpu_step(k, v, W, 1, tv, ts)
    assert loss == loss2 and all(np.array_equal(a, b) for a, b in zip(grads, grads2))
    ref = oracle.index_train(synth.to_bits(k), synth.to_bits(v), *W, tv.astype(np.float64), ts.astype(np.float64), 0.4, -0.3, act=1)
    assert abs(loss - ref[0]) <= 1e-3 * abs(ref[0])
    for got, want, name in zip(grads, ref[1:], ("dW_U", "db_U", "dW_V", "dW_S")):
        _check(got, want, name)
    gnorm2 = sum(float((g ** 2).sum()) for g in grads)
    step = 0.05 * loss / gnorm2                              # first-order decrease of 5 % of the loss
    W2 = [np.asarray(w - step * g.reshape(w.shape), dtype=np.float32) for w, g in zip(W, grads)]
    loss3, _ = _gpu_step(k, v, W2, 1, tv, ts)
    assert loss3 < loss


def test_train_argument_errors():
    hk, n, d_h = 1, 64, 64
    _, k, v = synth.qkv(1, 1, hk, n)
    k, v = k.cuda(), v.cuda()
    W = synth.indexer_weights(1, d_h, 1)
    w = vs.IndexerWeights(*[torch.from_numpy(x).cuda() for x in W], 0.0, 0.0, 1)
    t = torch.full((hk, n), 1.0 / n, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    g = [torch.zeros(s, dtype=torch.float32, device="cuda") for s in ((256, d_h), (d_h,), (d_h,), (d_h,))]
    ws = torch.empty(vs.index_train_workspace(hk, n, d_h), dtype=torch.uint8, device="cuda")
    with pytest.raises(vs.VsError) as e:
        vs.index_train_step(k, v, w, t, t, loss, *g, ws[:64])
    assert e.value.code == -3
    with pytest.raises(vs.VsError) as e:
        vs.index_train_step(k, v, w, t, t, loss, *g, ws, eps=0.0)
    assert e.value.code == -1
