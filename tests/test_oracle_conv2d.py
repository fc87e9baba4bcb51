"""Pins for the conv2d oracle: an independent im2col+matmul formulation on exact
integer data, delta kernels, valid-tap counts, stride/pad variants, torch float64."""
import numpy as np
import pytest
import torch

import oracle
from workloads import configs, rng


def _im2col_ref(x, w, stride, pad):
    """Independent formulation: pad explicitly, gather patches, one numpy matmul."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    sh, sw = stride
    ph, pw = pad
    xp = np.zeros((N, H + 2 * ph, W + 2 * pw, C))
    xp[:, ph:ph + H, pw:pw + W, :] = x
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    cols = np.empty((N, P, Q, R, S, C))
    for p in range(P):
        for q in range(Q):
            cols[:, p, q] = xp[:, p * sh:p * sh + R, q * sw:q * sw + S, :]
    return (cols.reshape(N * P * Q, R * S * C) @ w.reshape(K, R * S * C).T).reshape(N, P, Q, K)


@pytest.mark.parametrize("H,W,R,S,stride,pad", [
    (5, 7, 3, 3, (1, 1), (1, 1)), (5, 7, 1, 3, (1, 1), (0, 1)), (7, 5, 3, 1, (1, 1), (1, 0)),
    (8, 9, 3, 3, (2, 2), (1, 1)), (8, 9, 3, 3, (1, 1), (0, 0)), (9, 8, 5, 5, (2, 1), (2, 2)),
    (6, 6, 2, 2, (2, 2), (0, 0)), (4, 4, 3, 3, (1, 1), (2, 2)),
])
def test_matches_im2col_on_exact_integers(H, W, R, S, stride, pad):
    g = np.random.default_rng(H * 100 + W * 10 + R)
    x = g.integers(-4, 5, (2, H, W, 3)).astype(np.float64)
    w = g.integers(-4, 5, (4, R, S, 3)).astype(np.float64)
    y = oracle.conv2d(x, w, stride, pad)
    assert np.array_equal(y, _im2col_ref(x, w, stride, pad))


def test_centre_delta_is_identity():
    g = np.random.default_rng(0)
    C = 6
    x = g.standard_normal((2, 5, 7, C))
    w = np.zeros((C, 3, 3, C))
    w[np.arange(C), 1, 1, np.arange(C)] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, (1, 1), (1, 1)), x)


def test_corner_delta_shifts_down_right_with_zero_border():
    # w[k,0,0,c] = [k==c]  =>  y[p,q] = x[p-1,q-1], first row and column zero.
    g = np.random.default_rng(1)
    C = 4
    x = g.standard_normal((1, 5, 7, C))
    w = np.zeros((C, 3, 3, C))
    w[np.arange(C), 0, 0, np.arange(C)] = 1.0
    y = oracle.conv2d(x, w, (1, 1), (1, 1))
    expect = np.zeros_like(x)
    expect[:, 1:, 1:, :] = x[:, :-1, :-1, :]
    assert np.array_equal(y, expect)
    # the r index pairs with height: a delta at (r=0, s=2) shifts down and LEFT
    w2 = np.zeros((C, 3, 3, C))
    w2[np.arange(C), 0, 2, np.arange(C)] = 1.0
    y2 = oracle.conv2d(x, w2, (1, 1), (1, 1))
    expect2 = np.zeros_like(x)
    expect2[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    assert np.array_equal(y2, expect2)


def test_all_ones_counts_valid_taps():
    C, K = 64, 3
    y = oracle.conv2d(np.ones((1, 6, 8, C)), np.ones((K, 3, 3, C)), (1, 1), (1, 1))
    assert np.all(y[0, 1:-1, 1:-1] == 9 * C)          # 576 interior
    assert np.all(y[0, 0, 1:-1] == 6 * C) and np.all(y[0, 1:-1, -1] == 6 * C)   # 384 edge
    assert y[0, 0, 0, 0] == 4 * C and y[0, -1, -1, K - 1] == 4 * C             # 256 corner


def test_one_by_one_filter_is_a_gemm():
    g = np.random.default_rng(2)
    x = g.integers(-3, 4, (2, 4, 5, 8)).astype(np.float64)
    w = g.integers(-3, 4, (6, 1, 1, 8)).astype(np.float64)
    y = oracle.conv2d(x, w)
    c = oracle.gemm(x.reshape(-1, 8), w.reshape(6, 8), 40, 6, 8, b_col=True)
    assert np.array_equal(y.reshape(40, 6), c)


def test_against_torch_float64_on_workload_recipe():
    wl = configs.ConvWorkload(N=2, H=14, W=12, C=16, K=8)
    d = wl.make()
    x = rng.bf16_bits_to_f32(d["x_bf16"]).astype(np.float64)
    w = rng.bf16_bits_to_f32(d["w_bf16"]).astype(np.float64)
    y, ad = oracle.conv2d(x, w, (1, 1), (1, 1), want_absdot=True)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                                     torch.from_numpy(w).permute(0, 3, 1, 2), padding=1)
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.max(np.abs(y - ref)) < 1e-13
    assert np.allclose(ad, _im2col_ref(np.abs(x), np.abs(w), (1, 1), (1, 1)), rtol=1e-13)
    assert 0.0 <= x.min() and x.max() <= 1.0
