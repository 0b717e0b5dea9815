"""Pins for the budget / TopK oracle (Sec. "Adaptive Sparse Index Selection"): closed forms, a dyadic
hand example with a tie, a statistical law, and agreement with a plain fp64 sort + cumsum."""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def picked(idx, cnt, h=0):
    return idx[h, :cnt[h]].tolist()


def test_dyadic_hand_example():
    lines = [l.strip() for l in open(os.path.join(GOLD, "select_dyadic.txt")) if l.strip() and not l.startswith("#")]
    scores = np.array([[float(x) for x in lines[0].split()[1:]]], dtype=np.float32)
    for line in lines[1:]:
        tau, rest = line.split(":")
        want = [int(x) for x in rest.split()]
        idx, cnt, status, k = oracle.select(scores, mode=0, tau=float(tau))
        assert picked(idx, cnt) == want, (tau, picked(idx, cnt))
        assert k[0] == len(want) and status[0] == 0


@pytest.mark.parametrize("n,tau", [(1024, 0.9), (4096, 0.5), (256, 1.0), (64, 0.0), (2048, 0.85)])
def test_uniform_scores_closed_form(n, tau):
    """All scores 1/n (n a power of two: exact) => k = ceil(tau * n), lowest indices win every tie."""
    scores = np.full((2, n), 1.0 / n, dtype=np.float32)
    idx, cnt, status, k = oracle.select(scores, tau=tau)
    kk = math.ceil(tau * n)
    assert k.tolist() == [kk, kk]
    assert picked(idx, cnt, 1) == list(range(kk))


@pytest.mark.parametrize("r,tau", [(0.5, 0.9), (0.9, 0.9), (0.99, 0.85), (0.7, 0.999)])
def test_geometric_scores_closed_form(r, tau):
    """s_i proportional to r^i: top-k mass is (1 - r^k) / (1 - r^n), so k = ceil(log(1 - tau (1 - r^n)) / log r)."""
    n = 2000
    s = r ** np.arange(n, dtype=np.float64)
    s /= s.sum()
    want = math.ceil(math.log(1 - tau * (1 - r ** n)) / math.log(r))
    idx, cnt, _, k = oracle.select(s.astype(np.float32)[None], tau=tau)
    assert k[0] == want
    assert picked(idx, cnt) == list(range(want))
    # reversed order of the same scores: picks are the last `want` positions, emitted ascending
    idx, cnt, _, _ = oracle.select(s[::-1].astype(np.float32)[None], tau=tau)
    assert picked(idx, cnt) == list(range(n - want, n))


@pytest.mark.parametrize("std,tau,frac", [(3.0, 0.9, 0.0429), (2.0, 0.9, 0.2363), (3.0, 0.85, 0.0248), (3.0, 0.95, 0.0876)])
def test_gaussian_logits_fraction(std, tau, frac):
    """softmax of N(0, std^2) logits is log-normal: the mass above logit x is Phi(std - x/std), so the
    tau-mass set is the top Phi(z_tau - std) fraction.  Statistical pin, 10 % relative."""
    rng = np.random.default_rng(1)
    n = 1 << 18
    l = rng.standard_normal(n) * std
    s = np.exp(l - l.max())
    s /= s.sum()
    _, cnt, _, k = oracle.select(s.astype(np.float32)[None], tau=tau)
    assert abs(k[0] / n - frac) < 0.1 * frac, k[0] / n


@pytest.mark.parametrize("seed", range(6))
def test_integer_rule_matches_float_sort_cumsum(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(100, 5000))
    l = rng.standard_normal(n) * rng.uniform(0.5, 4.0)
    s = np.exp(l - l.max())
    s = (s / s.sum()).astype(np.float32)
    s[rng.integers(0, n, size=n // 10)] = s[rng.integers(0, n)]          # plant ties
    tau = float(rng.uniform(0.3, 0.99))
    order = np.lexsort((np.arange(n), -s.astype(np.float64)))
    cum = np.cumsum(s.astype(np.float64)[order])
    k_ref = int(np.searchsorted(cum, tau * cum[-1] * (1 - 1e-12), side="left")) + 1
    idx, cnt, status, k = oracle.select(s[None], tau=tau)
    assert abs(int(k[0]) - k_ref) <= 1                                    # 2^-40 quantisation of the masses
    assert picked(idx, cnt) == sorted(order[:k[0]].tolist())
    assert np.all(np.diff(idx[0, :cnt[0]]) > 0)


def test_fixed_k_forced_and_capacity():
    s = np.array([[0.05, 0.3, 0.05, 0.2, 0.05, 0.2, 0.1, 0.05]], dtype=np.float32)
    idx, cnt, st, k = oracle.select(s, mode=1, k_fixed=3)
    assert picked(idx, cnt) == [1, 3, 5] and st[0] == 0
    idx, cnt, st, k = oracle.select(s, mode=1, k_fixed=5)                 # ties among the 0.05s -> lowest index
    assert picked(idx, cnt) == [0, 1, 3, 5, 6]
    idx, cnt, st, k = oracle.select(s, mode=1, k_fixed=3, n_forced=2)      # union with {0,1}
    assert picked(idx, cnt) == [0, 1, 3, 5]
    idx, cnt, st, k = oracle.select(s, mode=1, k_fixed=100)
    assert picked(idx, cnt) == list(range(8)) and k[0] == 8
    # capacity: forced stay, best-ranked others fill the rest, overflow flagged
    idx, cnt, st, k = oracle.select(s, mode=1, k_fixed=5, n_forced=2, cap=3)
    assert picked(idx, cnt) == [0, 1, 3] and st[0] & 1
    idx, cnt, st, k = oracle.select(s, mode=0, tau=0.7, n_forced=1, cap=8)  # 0.3+0.2+0.2 = 0.7 -> {1,3,5} + {0}
    assert picked(idx, cnt) == [0, 1, 3, 5] and k[0] == 3 and st[0] == 0
    with pytest.raises(ValueError):
        oracle.select(s, n_forced=4, cap=3)


def test_bad_scores_are_flagged_not_fatal():
    s = np.array([[0.5, np.nan, -0.25, 0.25, -0.0, 0.25]], dtype=np.float32)
    idx, cnt, st, k = oracle.select(s, tau=0.75)
    assert picked(idx, cnt) == [0, 3] and st[0] & 2
    s = np.array([[2.0, 0.5, 0.5]], dtype=np.float32)                      # > 1 saturates to mass 2^40
    idx, cnt, st, k = oracle.select(s, tau=0.5)
    assert picked(idx, cnt) == [0] and st[0] & 4
    z = np.zeros((1, 16), dtype=np.float32)                                 # no mass at all: T = 0 -> nothing picked
    idx, cnt, st, k = oracle.select(z, tau=0.9, n_forced=1)
    assert picked(idx, cnt) == [0] and k[0] == 0
