"""Seeded synthetic inputs shaped like the paper's workloads (4B / 8B GQA layers: 32 query heads,
8 KV heads, head_dim 128).  They stand in for real prompts run through the backbone models, which
are not available; the structure follows the paper's description of real attention (heavy-hitter
columns, a strong near-diagonal band, discrete long-range offset bands).

This module holds input recipes only: no RoPE, no indexer, no selection, no attention.  It belongs to
neither the library nor the oracle: the tests, the benchmark and the smoke check feed both from here.
"""
import numpy as np
import torch

SEED_BASE = 2603 * 10 ** 4 + 4460          # + config number


def config_seed(config_no):
    return SEED_BASE + int(config_no)


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def normal(shape, seed):
    """fp32 N(0,1) tensor on the CPU from a seed."""
    return torch.randn(*shape, generator=_gen(seed), dtype=torch.float32)


def smooth_tokens(x, window=33):
    """Moving average over `window` consecutive innovations along the sequence axis, rescaled to unit
    variance: token j is correlated with tokens j-1 .. j-(window-1) (correlation 1 - lag/window)."""
    h, n, d = x.shape
    pad = torch.cat([x.new_zeros(h, 1, d), x], dim=1).cumsum(dim=1, dtype=torch.float64)
    lo = torch.clamp(torch.arange(n) - window + 1, min=0)
    s = pad[:, 1:, :] - pad[:, lo, :]
    return (s / np.sqrt(window)).to(torch.float32)


def qkv(seed, q_heads, kv_heads, n, local_structure=False, window=33):
    """Pre-RoPE Q, K, V as bf16 CPU tensors [heads, n, 128].  With local_structure, K and V are moving
    averages of white noise so that neighbouring tokens resemble each other."""
    q = normal((q_heads, n, 128), seed * 7 + 1)
    k = normal((kv_heads, n, 128), seed * 7 + 2)
    v = normal((kv_heads, n, 128), seed * 7 + 3)
    if local_structure:
        k = smooth_tokens(k, window)
        v = smooth_tokens(v, window)
    return q.to(torch.bfloat16), k.to(torch.bfloat16), v.to(torch.bfloat16)


def to_bits(t):
    """bf16 tensor (any device) -> numpy uint16 bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def from_bits(a, device="cpu"):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def heavy_hitter_plan(seed, kv_heads, n, count=16):
    """Shared unit direction u [128] and `count` distinct key positions per KV head."""
    g = _gen(seed * 7 + 4)
    u = torch.randn(128, generator=g, dtype=torch.float32)
    u = u / u.norm()
    cols = torch.stack([torch.randperm(n, generator=g)[:count].sort().values for _ in range(kv_heads)])
    return u, cols


def plant_heavy_hitters(q, k, u, cols, k_gain=4.0, q_gain=16.0):
    """Applied AFTER RoPE so that the planted columns attract every query regardless of distance:
    K[g, cols[g]] += k_gain * u and Q += (q_gain / sqrt(128)) * u, then back to bf16.  Works on CPU or GPU
    tensors (bf16 in, bf16 out)."""
    dev = k.device
    u = u.to(dev)
    kf = k.float()
    for g in range(k.shape[0]):
        kf[g, cols[g].to(dev)] += k_gain * u
    qf = q.float() + (q_gain / np.sqrt(128.0)) * u
    return qf.to(torch.bfloat16), kf.to(torch.bfloat16)


def fixed_lists(seed, n, n_sink=4, n_rand_v=60, n_local=64, n_rand_s=64, heads=1):
    """Config-1 style fixed mask: columns {0..n_sink-1} + random columns; offsets {0..n_local-1} + random
    offsets in [n_local, n).  Returns int32 (idx_v, cnt_v, idx_s, cnt_s), lists ascending."""
    rng = np.random.default_rng(seed)
    cap_v, cap_s = n_sink + n_rand_v, n_local + n_rand_s
    idx_v = np.zeros((heads, cap_v), dtype=np.int32)
    idx_s = np.zeros((heads, cap_s), dtype=np.int32)
    for h in range(heads):
        rv = rng.choice(np.arange(n_sink, n), size=n_rand_v, replace=False)
        rs = rng.choice(np.arange(n_local, n), size=n_rand_s, replace=False)
        idx_v[h] = np.sort(np.concatenate([np.arange(n_sink), rv]))
        idx_s[h] = np.sort(np.concatenate([np.arange(n_local), rs]))
    return idx_v, np.full(heads, cap_v, np.int32), idx_s, np.full(heads, cap_s, np.int32)


def structured_scores(seed, heads, n, n_planted=16, n_bands=6, band_width=48.0, white=False):
    """Seeded per-head score vectors for the fixed-budget config (each sums to 1, fp32):
    vertical = log-normal noise + sinks + planted heavy hitters; slash = decaying local band + a few
    Gaussian bands at long-range offsets + small noise.  white=True gives unstructured scores (the
    worst case for tile coverage)."""
    rng = np.random.default_rng(seed)
    a_v = np.empty((heads, n), dtype=np.float32)
    a_s = np.empty((heads, n), dtype=np.float32)
    t = np.arange(n, dtype=np.float64)
    for h in range(heads):
        lv = rng.standard_normal(n)
        ls = 0.3 * rng.standard_normal(n)
        if not white:
            lv[:4] += 8.0
            lv[rng.choice(np.arange(4, n), size=n_planted, replace=False)] += 6.0
            ls += 8.0 * np.exp(-t / (n / 48.0))
            for c in rng.uniform(0.05 * n, 0.95 * n, size=n_bands):
                ls += rng.uniform(4.0, 7.0) * np.exp(-0.5 * ((t - c) / band_width) ** 2)
        else:
            ls = rng.standard_normal(n)
        for l, a in ((lv, a_v), (ls, a_s)):
            e = np.exp(l - l.max())
            a[h] = (e / e.sum()).astype(np.float32)
    return a_v, a_s


# Down-projection gain that brings the logit spread of the default-initialised indexer (U(+-1/sqrt(fan_in)),
# GELU, d_h = 256) on unit-variance inputs to a standard deviation of about 3, the regime in which a 0.9
# cumulative threshold keeps a few percent of the positions.  Default init alone gives a spread of ~0.2 and
# hence almost uniform scores.  Measured once with the fp64 oracle; declared here as part of the recipe.
INDEXER_GAIN = {(256, 1): 14.0, (1024, 0): 14.0}


def indexer_weights(seed, d_h=256, act=1, gain=None):
    """Random-init VSIndexer parameters (numpy fp32): W_U [256, d_h], b_U [d_h], W_V [d_h], W_S [d_h]."""
    rng = np.random.default_rng(seed)
    bu = 1.0 / np.sqrt(256.0)
    bd = 1.0 / np.sqrt(float(d_h))
    if gain is None:
        gain = INDEXER_GAIN.get((d_h, act), 14.0)
    W_U = rng.uniform(-bu, bu, (256, d_h)).astype(np.float32)
    b_U = rng.uniform(-bu, bu, d_h).astype(np.float32)
    W_V = (gain * rng.uniform(-bd, bd, d_h)).astype(np.float32)
    W_S = (gain * rng.uniform(-bd, bd, d_h)).astype(np.float32)
    return W_U, b_U, W_V, W_S


def sample_rows(seed, n, first=64, last=64, rand=128):
    """Declared row sample for full-size parity: the first rows, the last rows and seeded uniform rows."""
    rng = np.random.default_rng(seed)
    first, last = min(first, n), min(last, n)
    mid = rng.choice(n, size=min(rand, n), replace=False)
    return np.unique(np.concatenate([np.arange(first), np.arange(n - last, n), mid])).astype(np.int64)


def score_structure_profile(seed, kv_heads, n, hh_cols, local_peak=12.0, n_bands=6, band_peak=(9.0, 12.0),
                            sink_peak=12.0, hh_peak=9.0):
    """Nominal logit boosts [kv_heads, n] (float64) that give the indexer's scores the structure the paper
    describes for real attention maps: for the slash direction a near-diagonal band that decays over
    ~n/128 offsets plus `n_bands` narrow long-range bands (width n/4096 .. n/2048) at seeded offsets; for the
    vertical direction the first four columns (sinks) and the planted heavy-hitter columns `hh_cols`."""
    rng = np.random.default_rng(seed * 7 + 5)
    t = np.arange(n, dtype=np.float64)
    d_s = np.zeros((kv_heads, n))
    d_v = np.zeros((kv_heads, n))
    for g in range(kv_heads):
        d_s[g] = local_peak * np.exp(-t / (n / 128.0))
        for _ in range(n_bands):
            c = rng.uniform(0.03 * n, 0.97 * n)
            w = rng.uniform(n / 4096.0, n / 2048.0)
            d_s[g] += rng.uniform(*band_peak) * np.exp(-0.5 * ((t - c) / w) ** 2)
        d_v[g, :min(4, n)] = sink_peak
        d_v[g, np.asarray(hh_cols[g])] = hh_peak
    return d_s, d_v


def plant_score_structure(k, v, W_U, W_V, W_S, d_s, d_v):
    """Adds, to token t of [K || V], d_s[t] * e_S + d_v[t] * e_V where e_S = W_U W_S / (0.5 |W_U W_S|^2) is the
    input direction whose unit multiple moves the slash logit by about one (first-order response of the
    two-layer net with a GELU / SiLU slope of about one half), likewise e_V for the vertical logit.  Applied to
    post-RoPE K and to V; bf16 in, bf16 out, any device.  A recipe for inputs only: it evaluates no score."""
    dev = k.device
    wu = torch.from_numpy(np.asarray(W_U, dtype=np.float64))
    e = []
    for wd in (W_S, W_V):
        d = wu @ torch.from_numpy(np.asarray(wd, dtype=np.float64))
        e.append((d / (0.5 * d.dot(d))).to(torch.float32).to(dev))
    a_s = torch.as_tensor(d_s, dtype=torch.float32, device=dev).unsqueeze(-1)
    a_v = torch.as_tensor(d_v, dtype=torch.float32, device=dev).unsqueeze(-1)
    add = a_s * e[0] + a_v * e[1]                       # [hk, n, 256]
    k2 = (k.float() + add[..., :128]).to(torch.bfloat16)
    v2 = (v.float() + add[..., 128:]).to(torch.bfloat16)
    return k2, v2
