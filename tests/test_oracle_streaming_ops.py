"""Pins for the oracle's RMS norm, mean along an axis and element-wise operators (the "rmsnorm",
"reducemean", "add", "mul", "relu" rows of the paper's operator table, Section 4.3): closed
forms, invariants and numpy second opinions."""
import numpy as np

import oracle


def test_rmsnorm_closed_forms():
    a, eps, D = 3.0, 1e-5, 64
    g = np.linspace(0.5, 1.5, D)
    # constant row: mean square a^2 -> y = a / sqrt(a^2 + eps) * gamma (no centring, unlike LayerNorm)
    y, r = oracle.rmsnorm(np.full((1, D), a), g, eps)
    np.testing.assert_allclose(r, 1 / np.sqrt(a * a + eps), rtol=1e-15)
    np.testing.assert_allclose(y[0], a / np.sqrt(a * a + eps) * g, rtol=1e-15)
    # alternating +-a has the same mean square
    x = a * (-1.0) ** np.arange(D)
    y, _ = oracle.rmsnorm(x[None], g, eps)
    np.testing.assert_allclose(y[0], x / np.sqrt(a * a + eps) * g, rtol=1e-15)
    # ramp 1..D: mean square (D+1)(2D+1)/6
    x = np.arange(1, D + 1, dtype=np.float64)
    _, r = oracle.rmsnorm(x[None], np.ones(D), 0.0)
    np.testing.assert_allclose(r, 1 / np.sqrt((D + 1) * (2 * D + 1) / 6.0), rtol=1e-15)


def test_rmsnorm_invariants_and_numpy():
    g = np.random.default_rng(1)
    x = g.standard_normal((7, 100)) * 3 + 1
    gamma = g.uniform(0.5, 1.5, 100)
    y, r = oracle.rmsnorm(x, gamma, 1e-6)
    np.testing.assert_allclose(y, x / np.sqrt((x * x).mean(1, keepdims=True) + 1e-6) * gamma, rtol=1e-13)
    # pre-affine output has mean square ms/(ms+eps)
    y1, _ = oracle.rmsnorm(x, np.ones(100), 1e-6)
    ms = (x * x).mean(1)
    np.testing.assert_allclose((y1 * y1).mean(1), ms / (ms + 1e-6), rtol=1e-12)
    # scale equivariance up to eps: rmsnorm(c x) = sign(c) rmsnorm(x) when eps = 0; a shift is NOT removed
    y0, _ = oracle.rmsnorm(x, gamma, 0.0)
    yc, _ = oracle.rmsnorm(-4.0 * x, gamma, 0.0)
    np.testing.assert_allclose(yc, -y0, rtol=1e-13)
    ys, _ = oracle.rmsnorm(x + 5.0, gamma, 0.0)
    assert np.max(np.abs(ys - y0)) > 0.1


def test_reduce_mean_both_axes():
    x = np.arange(12, dtype=np.float64).reshape(3, 4)        # rows 0..3, 4..7, 8..11
    np.testing.assert_array_equal(oracle.reduce_mean(x, 1), [1.5, 5.5, 9.5])
    np.testing.assert_array_equal(oracle.reduce_mean(x, 0), [4.0, 5.0, 6.0, 7.0])
    g = np.random.default_rng(2)
    x = g.standard_normal((37, 53))
    np.testing.assert_allclose(oracle.reduce_mean(x, 1), x.mean(1), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.reduce_mean(x, 0), x.mean(0), rtol=1e-13, atol=1e-15)
    # mean of a constant is the constant; linearity
    np.testing.assert_array_equal(oracle.reduce_mean(np.full((5, 8), 2.5), 0), np.full(8, 2.5))
    np.testing.assert_allclose(oracle.reduce_mean(3 * x + 1, 1), 3 * oracle.reduce_mean(x, 1) + 1, rtol=1e-12)


def test_eltwise_exact_cases():
    a = np.array([[1.0, -2.0, 0.0, 3.5], [-0.0, 7.0, -1e-30, 2.0]])
    b = np.array([[4.0, 5.0, -6.0, 0.5], [1.0, -7.0, 3.0, 0.25]])
    np.testing.assert_array_equal(oracle.eltwise(oracle.ELTWISE_ADD, a, b), a + b)
    np.testing.assert_array_equal(oracle.eltwise(oracle.ELTWISE_MUL, a, b), a * b)
    r = oracle.eltwise(oracle.ELTWISE_RELU, a)
    np.testing.assert_array_equal(r, [[1.0, 0.0, 0.0, 3.5], [0.0, 7.0, 0.0, 2.0]])
    assert not np.any(np.signbit(r))     # relu(-0.0) and relu(negative) are +0


def test_batchnorm_closed_forms_and_invariants():
    eps = 1e-5
    g = np.random.default_rng(6)
    N, C, H, W = 3, 4, 5, 6
    x = g.standard_normal((N, C, H, W)) * np.array([1.0, 3.0, 0.5, 2.0])[None, :, None, None] + np.array([0.0, 10.0, -4.0, 1e3])[None, :, None, None]
    gamma, beta = g.uniform(0.5, 1.5, C), g.standard_normal(C)
    y, m, r = oracle.batchnorm(x, gamma, beta, eps)
    # numpy second opinion (statistics over N, H, W per channel, biased variance)
    mu = x.mean(axis=(0, 2, 3)); var = x.var(axis=(0, 2, 3))
    np.testing.assert_allclose(m, mu, rtol=1e-13)
    np.testing.assert_allclose(r, 1 / np.sqrt(var + eps), rtol=1e-12)
    np.testing.assert_allclose(y, (x - mu[None, :, None, None]) / np.sqrt(var + eps)[None, :, None, None] * gamma[None, :, None, None]
                               + beta[None, :, None, None], rtol=1e-9, atol=1e-12)
    # pre-affine output: zero mean, variance var/(var+eps) per channel
    y1, _, _ = oracle.batchnorm(x, np.ones(C), np.zeros(C), eps)
    np.testing.assert_allclose(y1.mean(axis=(0, 2, 3)), 0.0, atol=1e-10)
    np.testing.assert_allclose(y1.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-10)
    # channels are independent: permuting them permutes the result
    p = np.array([2, 0, 3, 1])
    yp, mp, rp = oracle.batchnorm(x[:, p], gamma[p], beta[p], eps)
    np.testing.assert_array_equal(yp, y[:, p]); np.testing.assert_array_equal(mp, m[p])
    # constant channel -> beta; two-valued channel +-a -> +-a/sqrt(a^2+eps)*gamma + beta
    xc = np.full((2, 1, 3, 4), 7.0)
    yc, mc, _ = oracle.batchnorm(xc, np.array([1.3]), np.array([0.25]), eps)
    assert np.all(yc == 0.25) and mc[0] == 7.0
    xa = 2.0 * (-1.0) ** np.arange(24).reshape(2, 1, 3, 4)
    ya, _, ra = oracle.batchnorm(xa, np.array([1.5]), np.array([-1.0]), eps)
    np.testing.assert_allclose(ya, xa / np.sqrt(4.0 + eps) * 1.5 - 1.0, rtol=1e-15)
    # N and HW are pooled: moving data between the batch and spatial axes changes nothing
    x2 = x.reshape(N, C, H * W)
    y2, m2, _ = oracle.batchnorm(np.concatenate([x2[:, :, :15], x2[:, :, 15:]], axis=0).reshape(2 * N, C, 15), gamma, beta, eps)
    np.testing.assert_allclose(m2, m, rtol=1e-13)
