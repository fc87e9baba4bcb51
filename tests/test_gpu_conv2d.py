"""GPU parity: perf_conv2d (implicit-GEMM MFMA kernel and direct kernel) against the CPU
oracle. Tolerances as for the GEMM with K = R*S*C; bf16 outputs additionally allow one
bf16 rounding of the result."""
import numpy as np
import pytest

import oracle
from workloads import configs, rng
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def _bits(a):
    return rng.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _check(wl, y_bf16=True, stride=None, pad=None, variant=0):
    d = wl.make()
    stride = stride or (wl.stride, wl.stride)
    pad = pad or (wl.pad, wl.pad)
    y = G.run_conv2d(d["x_bf16"], d["w_bf16"], stride, pad, y_bf16=y_bf16, variant=variant)
    ref, ad = oracle.conv2d(oracle.widen(d["x_bf16"], True), oracle.widen(d["w_bf16"], True), stride, pad,
                            want_absdot=True)
    yg = P.bf16_to_f64(y) if y_bf16 else y
    P.assert_contraction_close(yg, ref, ad, wl.R * wl.S * wl.C, out_bf16=y_bf16)


def test_config5_recipe_two_images_full_compare():
    _check(configs.ConvWorkload(N=2))
    _check(configs.ConvWorkload(N=2), y_bf16=False)


@pytest.mark.parametrize("kw", [
    dict(N=1, H=5, W=7, C=64, K=128), dict(N=3, H=9, W=6, C=128, K=40), dict(N=1, H=12, W=12, C=64, K=130),
    dict(N=2, H=8, W=8, C=64, K=64, R=1, S=1, pad=0), dict(N=1, H=10, W=9, C=64, K=32, R=5, S=5, pad=2),
    dict(N=2, H=11, W=13, C=64, K=96, stride=2), dict(N=1, H=8, W=8, C=64, K=16, pad=0),
])
def test_mfma_path_shapes(kw):
    _check(configs.ConvWorkload(**kw))


@pytest.mark.parametrize("kw", [dict(N=2), dict(N=1, H=12, W=40), dict(N=3, H=33, W=35), dict(N=1, H=40, W=70, stride=2),
                                dict(N=5, pad=0), dict(N=1, H=3, W=32)])
@pytest.mark.parametrize("y_bf16", [True, False])
def test_weights_in_registers_kernel(kw, y_bf16):
    # ragged last blocks, odd and even block counts per workgroup, fewer workgroups than CUs,
    # stride 2, no padding
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(**kw), y_bf16=y_bf16, variant=perf.CONV_WREG)


@pytest.mark.parametrize("kw", [dict(N=2), dict(N=8), dict(N=16), dict(N=1, H=32, W=32), dict(N=4, H=58, W=58, pad=0),
                                dict(N=2, H=16, W=128), dict(N=1, H=64, W=40), dict(N=4, H=60, W=120)])
@pytest.mark.parametrize("y_bf16", [True, False])
def test_input_resident_kernel(kw, y_bf16):
    # ranges of 32 .. 196 pixels that start anywhere in a row (lanes wrap to the next row inside a
    # block), ragged last blocks, one block per workgroup, no padding, rows wider than the default,
    # 900 workgroups of one block because no larger range divides the image
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(**kw), y_bf16=y_bf16, variant=perf.CONV_WRES)


def test_input_resident_kernel_edge_shapes():
    # a single image row (two of the three patch rows lie outside the image), padding wider than
    # the filter's half width, different padding per axis, the narrowest rows the kernel takes
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(N=3, H=1, W=32), variant=perf.CONV_WRES)
    _check(configs.ConvWorkload(N=2, H=5, W=30, pad=2), variant=perf.CONV_WRES, y_bf16=False)
    _check(configs.ConvWorkload(N=1, H=34, W=32), pad=(0, 1), variant=perf.CONV_WRES)
    _check(configs.ConvWorkload(N=1, H=32, W=34), pad=(1, 0), variant=perf.CONV_WRES, y_bf16=False)


def test_input_resident_kernel_refuses_what_it_cannot_run():
    import torch
    import paper_2511_03586_amd as perf
    buf = torch.zeros(1 << 22, dtype=torch.int16, device="cuda")
    # stride 2; pixel ranges that would straddle images (33 x 35 outputs, ranges of 32); rows too wide for the LDS
    for n, h, w_, st in [(2, 56, 56, 2), (3, 33, 35, 1), (1, 32, 1024, 1)]:
        rc = perf.perf_conv2d_variant(buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), n, h, w_, 64, 128, 3, 3, st, st, 1, 1,
                                      perf.PERF_BF16, perf.PERF_BF16, perf.CONV_WRES, G.stream(), check=False)
        assert rc == perf.PERF_ERR_UNSUPPORTED


@pytest.mark.parametrize("kw", [dict(N=2), dict(N=8, K=64), dict(N=2, K=64), dict(N=4, K=256), dict(N=4, H=40, W=40),
                                dict(N=1, K=64), dict(N=8, H=28, W=32), dict(N=4, H=58, W=58, pad=0), dict(N=2, H=16, W=72),
                                dict(N=8, K=256), dict(N=4, K=512), dict(N=32, H=24, W=32, K=512)])
@pytest.mark.parametrize("y_bf16", [True, False])
def test_channel_slab_kernel(kw, y_bf16):
    # 1, 2, 4 and 8 slabs of 64 output channels; ranges that start anywhere in a row; ranges of 392 pixels
    # whose 10 or 11 input rows pass through the 8-row ring (its slots are reused inside a range) and of
    # 768 pixels (a whole image, 26 rows) through the 16-row ring of a narrow image; one-step and odd-step ranges, ragged last
    # blocks, no padding, the narrowest and widest rows the ring takes
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(**kw), y_bf16=y_bf16, variant=perf.CONV_WSPLIT)


def test_channel_slab_kernel_refuses_what_it_cannot_run():
    import torch
    import paper_2511_03586_amd as perf
    buf = torch.zeros(1 << 22, dtype=torch.int16, device="cuda")
    # stride 2; no range length divides 33 x 35 outputs; rows too wide for the ring; K not a multiple of 64;
    # rows too narrow for a fill load
    for n, h, w_, k, st in [(2, 56, 56, 128, 2), (3, 33, 35, 128, 1), (1, 16, 512, 128, 1), (2, 56, 56, 96, 1),
                            (2, 56, 24, 128, 1)]:
        rc = perf.perf_conv2d_variant(buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), n, h, w_, 64, k, 3, 3, st, st, 1, 1,
                                      perf.PERF_BF16, perf.PERF_BF16, perf.CONV_WSPLIT, G.stream(), check=False)
        assert rc == perf.PERF_ERR_UNSUPPORTED


@pytest.mark.parametrize("kw,y_bf16", [
    (dict(N=16, H=56, W=56, C=32, K=256), True),     # 784 tiles of 128 pixels x 128 channels
    (dict(N=32, H=56, W=56, C=32, K=48), True),      # 784 tiles of 128 x 64, ragged channels
    (dict(N=4, H=56, W=56, C=32, K=256), False),     # 392 tiles of 64 x 128
    (dict(N=2, H=56, W=56, C=64, K=64), True),       # 98 tiles of 64 x 64
])
def test_mfma_path_tile_shapes(kw, y_bf16):
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(**kw), y_bf16=y_bf16, variant=perf.CONV_MFMA)


def test_mfma_rectangular_filter_and_mixed_stride_pad():
    wl = configs.ConvWorkload(N=2, H=9, W=14, C=64, K=48, R=1, S=3)
    _check(wl, pad=(0, 1))
    wl = configs.ConvWorkload(N=1, H=14, W=9, C=64, K=48, R=3, S=1)
    _check(wl, pad=(1, 0), stride=(2, 1))


@pytest.mark.parametrize("kw", [
    dict(N=2, H=9, W=9, C=3, K=10, R=5, S=5, pad=2), dict(N=1, H=7, W=5, C=10, K=3, R=3, S=3, pad=1, stride=2),
    dict(N=1, H=6, W=6, C=72, K=8),
])
def test_direct_path_shapes(kw):
    _check(configs.ConvWorkload(**kw))
    _check(configs.ConvWorkload(**kw), y_bf16=False)


@pytest.mark.parametrize("kw", [
    dict(N=2, H=40, W=70, C=3, K=10, R=5, S=5, pad=2),      # two row tiles, two column tiles, ragged in both
    dict(N=1, H=33, W=64, C=3, K=20, R=5, S=5, pad=2),      # two blocks of 16 output channels
    dict(N=1, H=12, W=16, C=3, K=7, R=3, S=3, pad=1),       # odd channel count: element-wise stores
    dict(N=2, H=20, W=66, C=4, K=16, R=3, S=3, pad=0),      # 4 channels, no padding
    dict(N=1, H=9, W=10, C=3, K=10, R=5, S=5, pad=3),       # padding wider than the filter's half width
    dict(N=1, H=70, W=130, C=3, K=10, R=5, S=5, pad=2),     # three tiles each way
])
@pytest.mark.parametrize("y_bf16", [True, False])
def test_filter_row_per_mfma_kernel(kw, y_bf16):
    import paper_2511_03586_amd as perf
    _check(configs.ConvWorkload(**kw), y_bf16=y_bf16, variant=perf.CONV_ROWMFMA)


def test_filter_row_per_mfma_kernel_refuses_what_it_cannot_run():
    import torch
    import paper_2511_03586_amd as perf
    buf = torch.zeros(1 << 16, dtype=torch.int16, device="cuda")
    bad = [dict(C=3, R=5, S=5, W=9), dict(C=3, R=5, S=5, W=10, stride=2), dict(C=5, R=3, S=3, W=10), dict(C=3, R=3, S=5, W=10)]
    for kw in bad:                                           # W*C odd; stride 2; no instance for these filters
        c, r, s_, w_, st = kw["C"], kw["R"], kw["S"], kw["W"], kw.get("stride", 1)
        rc = perf.perf_conv2d_variant(buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), 1, 10, w_, c, 4, r, s_, st, st, 1, 1,
                                      perf.PERF_BF16, perf.PERF_BF16, perf.CONV_ROWMFMA, G.stream(), check=False)
        assert rc == perf.PERF_ERR_UNSUPPORTED


def test_small_channel_kernel_channel_blocks_and_fp32_operands():
    # C < 32 and at least 16384 output pixels: channel-blocked direct kernel; K = 37 needs three
    # blocks of 16 with a ragged last one
    _check(configs.ConvWorkload(N=1, H=130, W=128, C=5, K=37, R=3, S=3, pad=1))
    _check(configs.ConvWorkload(N=2, H=11, W=6, C=1, K=6, R=3, S=2, pad=1, stride=2), y_bf16=False, variant=3)
    _check(configs.ConvWorkload(N=2, H=9, W=9, C=3, K=10, R=5, S=5, pad=2), variant=3)
    g = np.random.default_rng(4)
    x = g.standard_normal((2, 7, 9, 4)).astype(np.float32)
    w = g.standard_normal((9, 3, 3, 4)).astype(np.float32)
    y = G.run_conv2d(x, w, (1, 1), (1, 1), xw_bf16=False, y_bf16=False, variant=3)
    ref, ad = oracle.conv2d(x.astype(np.float64), w.astype(np.float64), (1, 1), (1, 1), want_absdot=True)
    assert np.max(np.abs(y - ref) / np.maximum(ad, 1e-30)) <= 36 * 2.0 ** -23


@pytest.mark.parametrize("kw", [
    dict(N=2, H=9, W=11, C=40, K=48),                         # bf16, channel count no multiple of 32: the automatic choice
    dict(N=1, H=14, W=9, C=24, K=70, R=3, S=1, pad=0, stride=2),
    dict(N=3, H=20, W=20, C=16, K=130, R=5, S=5, pad=2),      # three channel tiles of 64, ragged
    dict(N=8, H=56, W=56, C=8, K=128),                        # 196 x 1 tiles of 128 x 128
])
def test_fp32_matrix_instruction_implicit_gemm(kw):
    import paper_2511_03586_amd as perf
    wl = configs.ConvWorkload(**kw)
    _check(wl, variant=perf.CONV_F32MFMA)
    _check(wl, y_bf16=False)                                  # routed there by the shape rules
    # fp32 operands: every product rounded once more than with bf16 operands (bound with K + 1)
    d = wl.make()
    x, w = rng.bf16_bits_to_f32(d["x_bf16"]) * np.float32(1.001), rng.bf16_bits_to_f32(d["w_bf16"]) * np.float32(0.999)
    for y_bf16 in (False, True):
        y = G.run_conv2d(x, w, (wl.stride, wl.stride), (wl.pad, wl.pad), xw_bf16=False, y_bf16=y_bf16)
        ref, ad = oracle.conv2d(x.astype(np.float64), w.astype(np.float64), (wl.stride, wl.stride), (wl.pad, wl.pad),
                                want_absdot=True)
        yg = P.bf16_to_f64(y) if y_bf16 else y
        P.assert_contraction_close(yg, ref, ad, wl.R * wl.S * wl.C + 1, out_bf16=y_bf16)


def test_delta_kernels_and_tap_counts_are_exact():
    C = 64
    x = rng.bf16_bits_to_f32(configs.ConvWorkload(N=1, H=5, W=7, C=C, K=C).make()["x_bf16"])
    w = np.zeros((C, 3, 3, C), np.float32)
    w[np.arange(C), 1, 1, np.arange(C)] = 1.0
    y = G.run_conv2d(_bits(x), _bits(w), (1, 1), (1, 1), y_bf16=False)
    assert np.array_equal(y, x)                                   # centre delta = identity
    w = np.zeros((C, 3, 3, C), np.float32)
    w[np.arange(C), 0, 2, np.arange(C)] = 1.0                      # tap (r=0, s=2): shift down and left
    y = G.run_conv2d(_bits(x), _bits(w), (1, 1), (1, 1), y_bf16=True)
    expect = np.zeros_like(x)
    expect[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    assert np.array_equal(rng.bf16_bits_to_f32(y), expect)
    ones = G.run_conv2d(_bits(np.ones((1, 6, 8, C))), _bits(np.ones((3, 3, 3, C))), (1, 1), (1, 1), y_bf16=False)
    assert np.all(ones[0, 1:-1, 1:-1] == 9 * C) and np.all(ones[0, 0, 1:-1] == 6 * C)
    assert ones[0, 0, 0, 0] == 4 * C and ones[0, -1, -1, 2] == 4 * C


def test_config5_full_size_sampled():
    """Batch 32 in the benchmark's launch configuration: images 0, 13 and 31 are recomputed
    by the oracle in full (borders included)."""
    wl = configs.CONFIG5
    d = wl.make()
    for y_bf16 in (True, False):
        y = G.run_conv2d(d["x_bf16"], d["w_bf16"], (1, 1), (1, 1), y_bf16=y_bf16)
        for n in (0, 13, 31):
            ref, ad = oracle.conv2d(oracle.widen(d["x_bf16"][n:n + 1], True), oracle.widen(d["w_bf16"], True),
                                    (1, 1), (1, 1), want_absdot=True)
            yg = P.bf16_to_f64(y[n:n + 1]) if y_bf16 else y[n:n + 1]
            P.assert_contraction_close(yg, ref, ad, 576, out_bf16=y_bf16)


def test_config5_full_size_every_entry_exact_integers():
    """Config 5's launch with small-integer activations (0..8) and weights (-8..8): all partial sums
    are integers below 2^24, exact in fp32 in any order, so every one of the 12.8M outputs must be
    bit-equal to the exact value (fp32 output) or to its single bf16 rounding (bf16 output). The
    exact value is an im2col + float64 matmul on the host, tied to the oracle on two whole images."""
    wl = configs.CONFIG5
    g = np.random.default_rng(505)
    x = g.integers(0, 9, (wl.N, wl.H, wl.W, wl.C)).astype(np.float32)
    w = g.integers(-8, 9, (wl.K, wl.R, wl.S, wl.C)).astype(np.float32)
    xp = np.zeros((wl.N, wl.H + 2, wl.W + 2, wl.C), np.float64)
    xp[:, 1:-1, 1:-1] = x
    wm = w.astype(np.float64).reshape(wl.K, -1).T                 # [(r, s, c), k]
    exact = np.empty((wl.N, wl.P, wl.Q, wl.K), np.float64)
    for n in range(wl.N):
        win = np.lib.stride_tricks.sliding_window_view(xp[n], (wl.R, wl.S), axis=(0, 1))   # [P, Q, C, R, S]
        cols = win.transpose(0, 1, 3, 4, 2).reshape(wl.P * wl.Q, -1)                       # [(p, q), (r, s, c)]
        exact[n] = (cols @ wm).reshape(wl.P, wl.Q, wl.K)
    for n in (0, 31):
        assert np.array_equal(oracle.conv2d(x[n:n + 1].astype(np.float64), w.astype(np.float64), (1, 1), (1, 1)),
                              exact[n:n + 1])
    y32 = G.run_conv2d(_bits(x), _bits(w), (1, 1), (1, 1), y_bf16=False)
    assert np.array_equal(y32.astype(np.float64), exact)
    y16 = G.run_conv2d(_bits(x), _bits(w), (1, 1), (1, 1), y_bf16=True)
    assert np.array_equal(y16, oracle.round_bf16(exact))


def test_deterministic():
    d = configs.ConvWorkload(N=4).make()
    a = G.run_conv2d(d["x_bf16"], d["w_bf16"], (1, 1), (1, 1))
    b = G.run_conv2d(d["x_bf16"], d["w_bf16"], (1, 1), (1, 1))
    assert np.array_equal(a, b)
