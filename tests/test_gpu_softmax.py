"""GPU parity: perf_softmax (through the C ABI) against the CPU oracle.
Tolerance: max relative error 1e-5 over outputs >= 1e-30 (absolute 1e-35 below), argmax
per row exact, fp32 arithmetic on both the wave-per-row and the workgroup-per-row paths."""
import numpy as np
import pytest

import oracle
from workloads import configs
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def _check(x, scale=1.0, **kw):
    y = G.run_softmax(x, scale, **kw)
    ref = oracle.softmax(x, float(np.float32(scale)))
    P.assert_softmax_close(y, ref)
    assert np.max(np.abs(y.astype(np.float64).sum(axis=1) - 1.0)) < 1e-5
    return y, ref


def test_config1_full_parity_and_argmax():
    x = configs.CONFIG1.make()["x"]
    y, ref = _check(x)
    P.assert_argmax_exact(y, x.astype(np.float64))
    assert np.array_equal(y.argmax(axis=1), ref.argmax(axis=1))


@pytest.mark.parametrize("rows,cols", [
    (1, 1), (3, 1), (7, 4), (5, 8), (33, 1000), (130, 512), (9, 256), (2, 260), (5, 2048), (6, 1028),
    (3, 2052), (4, 5), (11, 1023), (2, 12289), (3, 20000), (257, 96),
])
def test_shapes_cover_both_paths_and_tails(rows, cols):
    x = configs.SoftmaxWorkload(rows=rows, cols=cols).make()["x"]
    _check(x)


@pytest.mark.parametrize("rows,cols", [
    (300, 4096), (40, 16384), (600, 8192),   # four and sixteen waves per row, whole row in LDS; the row loop
    (3, 36864), (3, 36868), (2, 50000),      # at the LDS capacity, just beyond it, well beyond it (tail read twice)
    (2, 50001), (5, 2049),                   # element accesses
])
def test_rows_beyond_the_register_kernel(rows, cols):
    x = configs.SoftmaxWorkload(rows=rows, cols=cols).make()["x"]
    y, _ = _check(x)
    P.assert_argmax_exact(y, x.astype(np.float64))
    _check(x[:3], -0.5)
    _check(x[:3], inplace=True)


@pytest.mark.parametrize("scale", [0.125, -1.0, 0.0, 3.0])
def test_scale(scale):
    x = configs.SoftmaxWorkload(rows=19, cols=512).make()["x"]
    y, _ = _check(x, scale)
    _check(configs.SoftmaxWorkload(rows=3, cols=3001).make()["x"], scale)   # workgroup path
    if scale == 0.0:
        assert np.array_equal(y, np.full_like(y, 1.0 / 512))


def test_padded_rows_unaligned_base_and_inplace():
    x = configs.SoftmaxWorkload(rows=37, cols=200).make()["x"]
    _check(x, ldx=208, ldy=204)               # vector path with row padding
    _check(x, ldx=203, ldy=201)               # odd leading dimension -> workgroup path
    _check(x, offset=1)                       # base pointer only 4-byte aligned
    _check(x, inplace=True)
    _check(x, ldx=203, inplace=True)


def test_wide_dynamic_range():
    g = np.random.default_rng(11)
    x = g.uniform(-80.0, 0.0, (16, 1024)).astype(np.float32)
    x[:, 3] = 0.0
    _check(x)
    _check(x[:, :1000].copy() * 0.5 - 3.0, scale=2.0)
    big = (g.uniform(-1, 1, (4, 512)) * 1e38).astype(np.float32)     # differences overflow fp32
    y = G.run_softmax(big)
    assert np.isfinite(y).all() and np.max(np.abs(y.sum(axis=1) - 1.0)) < 1e-5


def test_shift_invariance_is_bit_exact_on_a_grid():
    g = np.random.default_rng(12)
    x = (g.integers(-8192, 8192, (32, 1024)) / 1024.0).astype(np.float32)   # multiples of 2^-10, |x| < 8
    y0 = G.run_softmax(x)
    y1 = G.run_softmax(x + np.float32(64.0))                                # exact in fp32
    assert np.array_equal(y0, y1)


def test_closed_forms_on_gpu():
    assert np.array_equal(G.run_softmax(np.full((3, 1024), -7.5, dtype=np.float32)),
                          np.full((3, 1024), 2.0 ** -10, dtype=np.float32))
    x = np.zeros((2, 512), dtype=np.float32)
    x[0, 77] = 104.0
    x[1, 500] = 200.0
    y = G.run_softmax(x)
    expect = np.zeros_like(x)
    expect[0, 77] = 1.0
    expect[1, 500] = 1.0
    assert np.array_equal(y, expect)
    y = G.run_softmax(np.log(np.array([[1.0, 2.0, 3.0, 4.0]], dtype=np.float32)))
    assert np.allclose(y, [[0.1, 0.2, 0.3, 0.4]], rtol=1e-6)


def test_deterministic():
    x = configs.SoftmaxWorkload(rows=512, cols=1024).make()["x"]
    assert np.array_equal(G.run_softmax(x), G.run_softmax(x))


def test_large_shapes_sampled_rows_and_row_sums():
    """Bench-size launches (262144x512 as in the attention workload, 131072x1024): every
    row must sum to 1; rows sampled across the whole grid are compared with the oracle."""
    import torch
    import paper_2511_03586_amd as perf
    for rows, cols, scale in [(262144, 512, 1.0), (131072, 1024, 0.125)]:
        base = configs.SoftmaxWorkload(rows=4096, cols=cols).make()["x"]
        xd = G.dev(base).repeat(rows // 4096, 1)
        xd += torch.arange(rows, device="cuda", dtype=torch.float32)[:, None] % 7   # rows differ across the grid
        yd = torch.empty_like(xd)
        perf.perf_softmax(xd.data_ptr(), yd.data_ptr(), rows, cols, cols, cols, perf.PERF_F32, perf.PERF_F32,
                          scale, G.stream())
        torch.cuda.synchronize()
        sums = yd.double().sum(dim=1)
        assert float((sums - 1.0).abs().max()) < 1e-5
        idx = np.unique(np.concatenate([np.arange(0, rows, 997), [rows - 1, rows - 2, rows - 5]]))
        xs = xd[torch.from_numpy(idx).cuda()].cpu().numpy()
        ys = yd[torch.from_numpy(idx).cuda()].cpu().numpy()
        P.assert_softmax_close(ys, oracle.softmax(xs, scale))
