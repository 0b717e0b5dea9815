"""Pins for the RoPE oracle (Appendix, "RoPE Matrix Representation" and "Derivation of Expectation")."""
import numpy as np
import pytest

import oracle
from brute import bits_to_f64, f32_to_bf16_bits


def test_single_plane_matrix_entries():
    """d = 2: theta_0 = 1, so position t rotates (1, 0) to (cos t, sin t) and (0, 1) to (-sin t, cos t)."""
    x = np.array([[[1.0, 0.0], [1.0, 0.0], [0.0, 1.0]]])
    y = oracle.rope_f64(x, pos0=3, theta_base=10000.0)
    np.testing.assert_allclose(y[0, 0], [np.cos(3.0), np.sin(3.0)], atol=1e-15)
    np.testing.assert_allclose(y[0, 1], [np.cos(4.0), np.sin(4.0)], atol=1e-15)
    np.testing.assert_allclose(y[0, 2], [-np.sin(5.0), np.cos(5.0)], atol=1e-15)


def test_frequencies_and_identity_at_zero():
    d, base = 8, 100.0
    x = np.zeros((1, 2, d))
    x[0, :, 0::2] = 1.0
    y = oracle.rope_f64(x, pos0=0, theta_base=base)
    np.testing.assert_array_equal(y[0, 0], x[0, 0])                      # t = 0 is the identity
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    np.testing.assert_allclose(y[0, 1, 0::2], np.cos(theta), atol=1e-15)
    np.testing.assert_allclose(y[0, 1, 1::2], np.sin(theta), atol=1e-15)


@pytest.mark.parametrize("pairing", [0, 1])
def test_orthogonal_and_relative(pairing):
    rng = np.random.default_rng(0)
    d, n = 16, 40
    q0, k0 = rng.standard_normal(d), rng.standard_normal(d)
    q = oracle.rope_f64(np.tile(q0, (1, n, 1)), theta_base=1e4, pairing=pairing)
    k = oracle.rope_f64(np.tile(k0, (1, n, 1)), theta_base=1e4, pairing=pairing)
    np.testing.assert_allclose(np.linalg.norm(q[0], axis=1), np.linalg.norm(q0), rtol=1e-14)
    P = q[0] @ k[0].T
    for o in range(-n + 1, n):                                           # Toeplitz: depends on m - n only
        diag = np.diagonal(P, -o)
        np.testing.assert_allclose(diag, diag[0], atol=1e-12)


def test_expected_score_closed_form():
    """(R(m) q) . (R(n) k) = sum_p a_p cos((m - n) theta_p) - b_p sin((m - n) theta_p) with the a_p, b_p of the
    appendix (interleaved planes)."""
    rng = np.random.default_rng(1)
    d, n, base = 32, 24, 1e6
    q0, k0 = rng.standard_normal(d), rng.standard_normal(d)
    q = oracle.rope_f64(np.tile(q0, (1, n, 1)), theta_base=base)
    k = oracle.rope_f64(np.tile(k0, (1, n, 1)), theta_base=base)
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    a = q0[0::2] * k0[0::2] + q0[1::2] * k0[1::2]
    b = -q0[0::2] * k0[1::2] + q0[1::2] * k0[0::2]
    for m in range(n):
        for t in range(n):
            want = np.sum(a * np.cos((m - t) * theta) - b * np.sin((m - t) * theta))
            np.testing.assert_allclose(q[0, m] @ k[0, t], want, atol=1e-12)


def test_half_split_is_a_permutation_of_interleaved():
    rng = np.random.default_rng(2)
    d, n = 8, 10
    x = rng.standard_normal((2, n, d))
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])      # interleaved -> half-split coordinates
    y0 = oracle.rope_f64(x, pos0=5, theta_base=50.0, pairing=0)
    y1 = oracle.rope_f64(x[..., perm], pos0=5, theta_base=50.0, pairing=1)
    np.testing.assert_allclose(y1, y0[..., perm], atol=1e-15)


def test_bf16_storage_rounds_once_to_nearest_even():
    rng = np.random.default_rng(3)
    x = f32_to_bf16_bits(rng.standard_normal((2, 300, 128)).astype(np.float32))
    y = oracle.rope_bf16(x, pos0=131072 - 300, theta_base=1e6)
    exact = oracle.rope_f64(bits_to_f64(x), pos0=131072 - 300, theta_base=1e6)
    got = bits_to_f64(y)
    # nearest: error at most half a bf16 ulp of the exact value
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 1e-30))) - 7)
    assert np.all(np.abs(got - exact) <= 0.5 * ulp + 1e-300)
    # ties to even on exact halves, and the conversion helper on the worked values
    assert oracle.f64_to_bf16([1.00390625, 1.01171875, -2.0, 0.0]).tolist() == [0x3F80, 0x3F82, 0xC000, 0]
    np.testing.assert_array_equal(oracle.f64_to_bf16(bits_to_f64(x)), x)  # round trip is exact
