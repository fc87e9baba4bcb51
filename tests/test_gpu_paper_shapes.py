"""GPU parity at the shapes of the paper's own operator table (Section 4.3: softmax 24576x512,
layernorm 16384x1024 and 4096x4096, matmul 768x1024x1024, bmm 192x256x128x256, conv
8x64x64x56x56x3 and 8x10x3x512x512x5) with this repository's input recipes. Outputs are
computed in full on the GPU and compared with the oracle on sampled rows / matrices / images."""
import numpy as np
import pytest

import oracle
from workloads import configs, rng
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_softmax_24576x512():
    x = configs.PAPER_SOFTMAX.make()["x"]
    y = G.run_softmax(x)
    np.testing.assert_allclose(y.astype(np.float64).sum(1), 1.0, atol=1e-5)
    rows = np.arange(0, x.shape[0], 97)
    P.assert_softmax_close(y[rows], oracle.softmax(x[rows].astype(np.float64)))
    P.assert_argmax_exact(y[rows], x[rows].astype(np.float64))


@pytest.mark.parametrize("wl", [configs.PAPER_LAYERNORM_1, configs.PAPER_LAYERNORM_2], ids=["16384x1024", "4096x4096"])
def test_layernorm_fp32(wl):
    d = wl.make()
    x = rng.bf16_bits_to_f32(d["x_bf16"])          # fp32 tensor holding the recipe's values
    y, mean, rstd = G.run_layernorm(x, d["gamma"], d["beta"], wl.eps, False, False, False)
    rows = np.arange(0, wl.rows, 61)
    ref, mref, rref = oracle.layernorm(x[rows].astype(np.float64), d["gamma"], d["beta"], float(np.float32(wl.eps)))
    rms = np.sqrt(np.mean(ref ** 2, axis=1, keepdims=True))
    assert np.max(np.abs(y[rows] - ref) / np.maximum(np.abs(ref), rms)) <= 1e-5
    assert np.max(np.abs(mean[rows] - mref) / np.maximum(np.abs(mref), 1e-3)) <= 1e-5
    assert np.max(np.abs(rstd[rows] - rref) / rref) <= 1e-5


def test_matmul_768x1024x1024():
    wl = configs.PAPER_MATMUL
    d = wl.make()
    c = G.run_gemm(d["a_bf16"], d["b_bf16"], wl.M, wl.N, wl.K)[0]
    ad, bd = oracle.widen(d["a_bf16"], True), oracle.widen(d["b_bf16"], True)
    P.assert_contraction_close(c, oracle.gemm(ad, bd, wl.M, wl.N, wl.K, b_col=True),
                               oracle.gemm_absdot(ad, bd, wl.M, wl.N, wl.K, b_col=True), wl.K)


def test_bmm_192x256x128x256():
    wl, batch = configs.PAPER_BMM, configs.PAPER_BMM_BATCH
    d = wl.make()
    a = np.stack([np.roll(d["a_bf16"], i, axis=0) for i in range(batch)])
    b = np.stack([np.roll(d["b_bf16"], -i, axis=0) for i in range(batch)])
    c = G.run_gemm(a, b, wl.M, wl.N, wl.K, batch=batch)
    for i in (0, 1, 95, 191):
        ad, bd = oracle.widen(a[i], True), oracle.widen(b[i], True)
        P.assert_contraction_close(c[i], oracle.gemm(ad, bd, wl.M, wl.N, wl.K, b_col=True),
                                   oracle.gemm_absdot(ad, bd, wl.M, wl.N, wl.K, b_col=True), wl.K)


@pytest.mark.parametrize("wl,images", [(configs.PAPER_CONV_2, (0, 7)), (configs.PAPER_CONV_1, (3,))],
                         ids=["8x64x64x56x56x3", "8x10x3x512x512x5"])
def test_conv(wl, images):
    d = wl.make()
    y = G.run_conv2d(d["x_bf16"], d["w_bf16"], (wl.stride, wl.stride), (wl.pad, wl.pad), y_bf16=False)
    wd = oracle.widen(d["w_bf16"], True)
    for n in images:
        ref, ad = oracle.conv2d(oracle.widen(d["x_bf16"][n:n + 1], True), wd, (wl.stride, wl.stride),
                                (wl.pad, wl.pad), want_absdot=True)
        P.assert_contraction_close(y[n:n + 1], ref, ad, wl.R * wl.S * wl.C)


def _f32_bound_ok(c, ref, absdot, K):
    """fp32 operands: every product is rounded once (2^-24 relative) before it is accumulated in fp32
    in some order, so |err| <= (K + 1) 2^-23 sum|a||b| whatever the order; contract gate 2e-2 with the
    rms floor as for the bf16 contractions."""
    gate, _ = P.contraction_errors(c, ref, absdot)
    assert gate <= 2e-2
    assert np.all(np.abs(c.astype(np.float64) - ref) <= (K + 1) * 2.0 ** -23 * absdot + 2.0 ** -24 * np.abs(ref))
    return gate


def test_matmul_and_bmm_fp32_operands():
    """The table states no dtype: the same shapes with fp32 operands (the recipe's values before the
    bf16 rounding) through the fp32 matrix-instruction kernel, every entry against the oracle."""
    wl = configs.PAPER_MATMUL
    a = rng.uniform(rng.tensor_seed(wl.config, 0), (wl.M, wl.K), -1.0, 1.0)
    b = rng.uniform(rng.tensor_seed(wl.config, 1), (wl.N, wl.K), -1.0, 1.0)
    c = G.run_gemm(a, b, wl.M, wl.N, wl.K, ab_bf16=False)[0]
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    _f32_bound_ok(c, oracle.gemm(a64, b64, wl.M, wl.N, wl.K, b_col=True), oracle.gemm_absdot(a64, b64, wl.M, wl.N, wl.K, b_col=True), wl.K)
    wl, batch = configs.PAPER_BMM, configs.PAPER_BMM_BATCH
    a = rng.uniform(rng.tensor_seed(wl.config, 0), (batch, wl.M, wl.K), -1.0, 1.0)
    b = rng.uniform(rng.tensor_seed(wl.config, 1), (batch, wl.N, wl.K), -1.0, 1.0)
    c = G.run_gemm(a, b, wl.M, wl.N, wl.K, batch=batch, ab_bf16=False)
    for i in (0, 1, 95, 191):
        a64, b64 = a[i].astype(np.float64), b[i].astype(np.float64)
        _f32_bound_ok(c[i], oracle.gemm(a64, b64, wl.M, wl.N, wl.K, b_col=True),
                      oracle.gemm_absdot(a64, b64, wl.M, wl.N, wl.K, b_col=True), wl.K)


@pytest.mark.parametrize("M,N,K,a_col,b_col", [(130, 70, 33, False, True), (64, 64, 16, True, False), (257, 129, 65, False, False),
                                               (1, 1, 1, False, True), (300, 200, 100, True, True), (513, 260, 40, False, True)])
def test_fp32_matrix_instruction_kernel_layouts_and_tails(M, N, K, a_col, b_col):
    g = np.random.default_rng(M + N + K)
    a = g.standard_normal((K, M) if a_col else (M, K)).astype(np.float32)
    b = g.standard_normal((N, K) if b_col else (K, N)).astype(np.float32)
    c = G.run_gemm(a, b, M, N, K, a_col=a_col, b_col=b_col, alpha=0.75, ab_bf16=False)[0]
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    ref = oracle.gemm(a64, b64, M, N, K, a_col=a_col, b_col=b_col, alpha=0.75)
    absdot = 0.75 * oracle.gemm_absdot(a64, b64, M, N, K, a_col=a_col, b_col=b_col)
    _f32_bound_ok(c, ref, absdot, K)
    # exact integers: bit equality in any order
    ai = g.integers(-8, 9, a.shape).astype(np.float32)
    bi = g.integers(-8, 9, b.shape).astype(np.float32)
    ci = G.run_gemm(ai, bi, M, N, K, a_col=a_col, b_col=b_col, ab_bf16=False)[0]
    assert np.array_equal(ci.astype(np.float64), oracle.gemm(ai, bi, M, N, K, a_col=a_col, b_col=b_col))


@pytest.mark.parametrize("wl,images", [(configs.PAPER_CONV_2, (5,)), (configs.PAPER_CONV_1, (0,))],
                         ids=["8x64x64x56x56x3", "8x10x3x512x512x5"])
def test_conv_fp32_operands(wl, images):
    x = rng.uniform(rng.tensor_seed(wl.config, 0), (wl.N, wl.H, wl.W, wl.C), 0.0, 1.0)
    w = rng.normal(rng.tensor_seed(wl.config, 1), (wl.K, wl.R, wl.S, wl.C), 0.0, 2.0 / (wl.R * wl.S * wl.C))
    y = G.run_conv2d(x, w, (wl.stride, wl.stride), (wl.pad, wl.pad), xw_bf16=False, y_bf16=False)
    for n in images:
        ref, ad = oracle.conv2d(x[n:n + 1].astype(np.float64), w.astype(np.float64), (wl.stride, wl.stride),
                                (wl.pad, wl.pad), want_absdot=True)
        _f32_bound_ok(y[n:n + 1], ref, ad, wl.R * wl.S * wl.C)
