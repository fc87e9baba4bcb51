"""Pins for the LayerNorm oracle (closed forms, invariants, torch float64)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import configs, rng


def _small():
    d = configs.LayerNormWorkload(rows=32, cols=4096).make()
    return rng.bf16_bits_to_f32(d["x_bf16"]), d["gamma"], d["beta"]


def test_pre_affine_zero_mean_unit_variance():
    x, _, _ = _small()
    D = x.shape[1]
    eps = 1e-5
    y, mean, rstd = oracle.layernorm(x, np.ones(D), np.zeros(D), eps)
    assert np.max(np.abs(y.mean(axis=1))) < 1e-12
    var = x.astype(np.float64).var(axis=1)          # numpy's biased variance
    assert np.allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    assert np.allclose(mean, x.astype(np.float64).mean(axis=1), rtol=1e-13)
    assert np.allclose(rstd, 1.0 / np.sqrt(var + eps), rtol=1e-13)


def test_constant_row_returns_beta():
    D = 1024
    beta = np.linspace(-1, 1, D)
    y, mean, rstd = oracle.layernorm(np.full((2, D), 3.25), np.full(D, 1.7), beta, 1e-5)
    assert np.array_equal(y, np.stack([beta, beta]))
    assert np.array_equal(mean, [3.25, 3.25])
    assert np.allclose(rstd, 1.0 / np.sqrt(1e-5), rtol=1e-15)


def test_alternating_row_closed_form():
    D, a, eps = 512, 2.5, 1e-5
    x = np.tile([a, -a], D // 2)[None, :]
    gamma = np.linspace(0.5, 1.5, D)
    beta = np.linspace(-0.3, 0.3, D)
    y, mean, rstd = oracle.layernorm(x, gamma, beta, eps)
    assert mean[0] == 0.0
    assert rstd[0] == pytest.approx(1.0 / np.sqrt(a * a + eps), rel=1e-15)
    assert np.allclose(y[0], x[0] / np.sqrt(a * a + eps) * gamma + beta, rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("D", [7, 64, 4096])
def test_ramp_distinguishes_biased_variance(D):
    x = np.arange(D, dtype=np.float64)[None, :]
    _, mean, rstd = oracle.layernorm(x, np.ones(D), np.zeros(D), 0.0)
    assert mean[0] == pytest.approx((D - 1) / 2.0, rel=1e-15)
    biased = (D * D - 1) / 12.0
    unbiased = biased * D / (D - 1)
    assert 1.0 / rstd[0] ** 2 == pytest.approx(biased, rel=1e-13)
    assert abs(1.0 / rstd[0] ** 2 - unbiased) / unbiased > 1e-5


def test_affine_equivariance():
    x, gamma, beta = _small()
    x = x[:4].astype(np.float64)
    y0, _, _ = oracle.layernorm(x, gamma, beta, 0.0)
    y1, _, _ = oracle.layernorm(3.0 * x + 11.0, gamma, beta, 0.0)
    y2, _, _ = oracle.layernorm(-2.0 * x + 1.0, gamma, beta, 0.0)
    b = beta.astype(np.float64)
    assert np.allclose(y1, y0, rtol=1e-10, atol=1e-10)
    assert np.allclose(y2 - b, -(y0 - b), rtol=1e-10, atol=1e-10)


def test_large_offset_small_variance_is_stable():
    # mean 1e3, variance 1e-2: E[x^2]-E[x]^2 in fp32 would lose everything; the
    # two-pass definition must recover the variance to near double accuracy.
    g = np.random.default_rng(5)
    x = (1000.0 + 0.1 * g.standard_normal((4, 2048))).astype(np.float32)
    _, mean, rstd = oracle.layernorm(x, np.ones(2048), np.zeros(2048), 0.0)
    xd = x.astype(np.float64)
    assert np.allclose(mean, xd.mean(axis=1), rtol=1e-14)
    assert np.allclose(1.0 / rstd ** 2, ((xd - xd.mean(axis=1, keepdims=True)) ** 2).mean(axis=1), rtol=1e-10)


def test_against_torch_float64():
    x, gamma, beta = _small()
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (x.shape[1],),
                                         torch.from_numpy(gamma).double(),
                                         torch.from_numpy(beta).double(), eps=1e-5).numpy()
    y, _, _ = oracle.layernorm(x, gamma, beta, 1e-5)
    assert np.max(np.abs(y - ref)) < 1e-12


def test_round_bf16_is_single_rne():
    # exact bf16 values are fixed points; halfway cases go to even; a value that a
    # double->float->bf16 chain would double-round is rounded correctly.
    exact = np.array([1.0, -2.5, 0.15625, 3.3895313892515355e38, 2.0 ** -133, 0.0])
    bits = oracle.round_bf16(exact)
    assert np.array_equal(rng.bf16_bits_to_f32(bits).astype(np.float64), exact)
    # 1 + 2^-8 is halfway between 1 and 1+2^-7 -> even (1.0); 1+3*2^-8 -> 1+2^-6
    assert rng.bf16_bits_to_f32(oracle.round_bf16(np.array([1 + 2.0 ** -8])))[0] == 1.0
    assert rng.bf16_bits_to_f32(oracle.round_bf16(np.array([1 + 3 * 2.0 ** -8])))[0] == 1 + 2.0 ** -6
    # just above halfway by less than fp32 resolution: float() would round it to the tie
    v = 1 + 2.0 ** -8 + 2.0 ** -40
    assert rng.bf16_bits_to_f32(oracle.round_bf16(np.array([v])))[0] == 1 + 2.0 ** -7
    assert np.float32(v) == np.float32(1 + 2.0 ** -8)
    # agreement with torch's fp32->bf16 conversion on fp32-representable inputs
    g = np.random.default_rng(3)
    f = (g.standard_normal(20000) * np.exp(g.uniform(-30, 30, 20000))).astype(np.float32)
    t = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_bf16(f.astype(np.float64)), t)
    assert np.array_equal(rng.f32_to_bf16_bits(f), t)
