"""Dense n x n brute force of masked attention in numpy (tiny n only).

Independent of ``oracle/``: it materialises the mask matrix from the mask equation of
Sec. "Linear-Complexity Mask Construction" (plus causality), adds it to the scaled scores as in
Sec. "Sparse Attention Formulation", and applies a row softmax and a matmul.
"""
import numpy as np


def bits_to_f64(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even truncation of fp32 to bf16 bit patterns (finite inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def vs_mask(n, I_v, I_s, causal=True):
    I_v, I_s = set(int(x) for x in I_v), set(int(x) for x in I_s)
    M = np.full((n, n), -np.inf)
    for i in range(n):
        for j in range(n):
            if causal and j > i:
                continue
            if j in I_v or (i - j) in I_s:
                M[i, j] = 0.0
    return M


def masked_attention(q, k, v, M, scale):
    """q, k, v: [n, d] float64; M: [n, n] of {0, -inf}.  Rows with no live key give zeros."""
    P = q @ k.T * scale + M
    out = np.zeros_like(v, dtype=np.float64)
    lse = np.full(q.shape[0], -np.inf)
    for i in range(q.shape[0]):
        row = P[i]
        if not np.isfinite(row).any():
            continue
        m = row[np.isfinite(row)].max()
        e = np.where(np.isfinite(row), np.exp(row - m), 0.0)
        z = e.sum()
        out[i] = (e / z) @ v
        lse[i] = m + np.log(z)
    return out, lse
