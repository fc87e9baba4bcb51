"""GPU parity: perf_rmsnorm, perf_reduce_mean, perf_eltwise against the CPU oracle.
Tolerances: fp32 results of reductions 1e-5 relative (denominator floored at the RMS of the
quantity), bf16 results within 1 bf16 ulp of the oracle's single rounding; element-wise fp32
add / mul / relu are correctly rounded, hence bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_03586_amd as perf
from workloads import rng
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def _bf16(a):
    return rng.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _run_rmsnorm(x, gamma, eps, x_bf16, p_bf16, y_bf16, ldx=None, ldy=None, inplace=False):
    rows, cols = x.shape
    ldx = ldx or cols
    ldy = ldx if inplace else (ldy or cols)
    xb = np.zeros((rows, ldx), dtype=x.dtype); xb[:, :cols] = x
    xd = G.dev(xb.ravel())
    yd = xd if inplace else torch.zeros(rows * ldy, dtype=torch.int16 if y_bf16 else torch.float32, device="cuda")
    gd = G.dev(gamma)
    rd = torch.zeros(rows, dtype=torch.float32, device="cuda")
    perf.perf_rmsnorm(xd.data_ptr(), gd.data_ptr(), yd.data_ptr(), rd.data_ptr(), rows, cols, ldx, ldy, eps,
                      G.dt(x_bf16), G.dt(p_bf16), G.dt(y_bf16), G.stream())
    torch.cuda.synchronize()
    y = G.host(yd, y_bf16).reshape(rows, ldy)
    if not inplace:
        assert np.all(y[:, cols:] == 0), "kernel wrote into the row padding"
    return y[:, :cols].copy(), rd.cpu().numpy()


def _check_rmsnorm(rows, cols, x_bf16=True, p_bf16=False, y_bf16=True, seed=0, **kw):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((rows, cols)) * np.sqrt(3.0) + 1.0).astype(np.float32)
    gamma = g.uniform(0.5, 1.5, cols).astype(np.float32)
    xs = _bf16(x) if x_bf16 else x
    gs = _bf16(gamma) if p_bf16 else gamma
    y, r = _run_rmsnorm(xs, gs, 1e-5, x_bf16, p_bf16, y_bf16, **kw)
    ref, rref = oracle.rmsnorm(oracle.widen(xs, x_bf16), oracle.widen(gs, p_bf16), float(np.float32(1e-5)))
    assert np.max(np.abs(r - rref) / rref) <= 1e-5
    if y_bf16:
        got, want = P.bf16_to_f64(y), P.bf16_to_f64(oracle.round_bf16(ref))
        diff = np.abs(got - want)
        assert np.all(diff <= 2.0 ** -7 * np.maximum(np.abs(ref), 2.0 ** -7))
        assert np.mean(got == want) >= 0.999
    else:
        rms = np.sqrt(np.mean(ref ** 2, axis=1, keepdims=True))
        assert np.max(np.abs(y - ref) / np.maximum(np.abs(ref), rms)) <= 1e-5


@pytest.mark.parametrize("rows,cols", [(3072, 4096), (64, 1024), (5, 8), (33, 1000), (7, 8192), (9, 520), (2, 9000), (3, 7)])
def test_rmsnorm_bf16_shapes(rows, cols):
    _check_rmsnorm(rows, cols)


def test_rmsnorm_rows_beyond_the_register_kernel():
    _check_rmsnorm(200, 16384)                                   # four waves per row, row in LDS
    _check_rmsnorm(20, 32768, p_bf16=True)                       # sixteen waves per row
    _check_rmsnorm(3, 40000, x_bf16=False, y_bf16=False)         # beyond the LDS: the tail is read again
    _check_rmsnorm(2, 80000, y_bf16=False)
    _check_rmsnorm(5, 16384, inplace=True)
    _check_rmsnorm(5, 16384, ldx=16392, ldy=16400)


def test_rmsnorm_dtypes_padding_inplace():
    _check_rmsnorm(40, 2048, x_bf16=False, y_bf16=False)
    _check_rmsnorm(40, 4096, x_bf16=False, y_bf16=False)        # 16 chunks of fp32 per lane
    _check_rmsnorm(16, 512, x_bf16=False, p_bf16=True, y_bf16=True)
    _check_rmsnorm(16, 768, x_bf16=True, p_bf16=True, y_bf16=False)
    _check_rmsnorm(12, 256, ldx=264, ldy=272)
    _check_rmsnorm(12, 256, ldx=264, inplace=True)
    _check_rmsnorm(6, 250, x_bf16=False, y_bf16=False, ldx=251, ldy=253)   # block kernel: nothing aligned


def test_rmsnorm_closed_forms_on_gpu():
    D = 1024
    x = np.full((2, D), 3.0, np.float32); x[1] *= (-1.0) ** np.arange(D)
    y, r = _run_rmsnorm(x, np.ones(D, np.float32), 0.0, False, False, False)
    assert np.all(r == np.float32(1 / 3.0)) or np.max(np.abs(r - 1 / 3.0)) <= 1e-7
    np.testing.assert_allclose(y, np.sign(x), rtol=2e-7)


def _run_mean(x, axis, x_bf16, y_bf16, ldx=None, ws=False):
    rows, cols = x.shape
    ldx = ldx or cols
    xb = np.zeros((rows, ldx), dtype=x.dtype); xb[:, :cols] = x
    xd = G.dev(xb.ravel())
    n = rows if axis == 1 else cols
    yd = torch.zeros(n, dtype=torch.int16 if y_bf16 else torch.float32, device="cuda")
    if ws:
        nbytes = perf.perf_reduce_mean_workspace_bytes(rows, cols, axis, G.dt(x_bf16))
        assert nbytes >= 0
        # scratch with junk in it, a guard word behind it
        wd = torch.full((nbytes // 4 + 1,), float("nan"), dtype=torch.float32, device="cuda")
        perf.perf_reduce_mean_ws(xd.data_ptr(), yd.data_ptr(), wd.data_ptr() if nbytes else None, rows, cols, ldx, axis,
                                 G.dt(x_bf16), G.dt(y_bf16), G.stream())
        torch.cuda.synchronize()
        assert bool(torch.isnan(wd[-1]))  # nothing written past the stated size
    else:
        perf.perf_reduce_mean(xd.data_ptr(), yd.data_ptr(), rows, cols, ldx, axis, G.dt(x_bf16), G.dt(y_bf16), G.stream())
        torch.cuda.synchronize()
    return G.host(yd, y_bf16)


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (100, 1000), (1, 1), (3, 5), (257, 96), (64, 20000), (5000, 32), (70, 33)])
@pytest.mark.parametrize("axis", [0, 1])
def test_reduce_mean_fp32(rows, cols, axis):
    g = np.random.default_rng(rows + cols + axis)
    x = (g.standard_normal((rows, cols)) * 2 + 0.5).astype(np.float32)
    y = _run_mean(x, axis, False, False)
    ref = oracle.reduce_mean(x.astype(np.float64), axis)
    floor = np.sqrt(np.mean(x.astype(np.float64) ** 2))
    assert np.max(np.abs(y - ref) / np.maximum(np.abs(ref), floor)) <= 1e-5


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (100, 1000), (1, 4), (3, 8), (257, 96), (64, 20000), (5000, 32),
                                       (16384, 1024), (70, 33), (33, 260)])
@pytest.mark.parametrize("axis", [0, 1])
def test_reduce_mean_with_workspace_fp32(rows, cols, axis):
    g = np.random.default_rng(rows + cols + axis)
    x = (g.standard_normal((rows, cols)) * 2 + 0.5).astype(np.float32)
    y = _run_mean(x, axis, False, False, ws=True)
    ref = oracle.reduce_mean(x.astype(np.float64), axis)
    floor = np.sqrt(np.mean(x.astype(np.float64) ** 2))
    assert np.max(np.abs(y - ref) / np.maximum(np.abs(ref), floor)) <= 1e-5


def test_reduce_mean_with_workspace_bf16_padded_exact_and_reproducible():
    g = np.random.default_rng(4)
    x = (g.standard_normal((300, 264)) + 1).astype(np.float32)
    xb = _bf16(x)
    y = _run_mean(xb, 0, True, True, ldx=272, ws=True)
    ref = oracle.reduce_mean(oracle.widen(xb, True), 0)
    assert np.all(np.abs(P.bf16_to_f64(y) - ref) <= 2.0 ** -8 * np.maximum(np.abs(ref), 2.0 ** -7) + 1e-5)
    y32 = _run_mean(xb, 0, True, False, ldx=272, ws=True)
    assert np.max(np.abs(y32 - ref)) <= 1e-5 * 1.5
    xi = g.integers(-8, 9, (1024, 512)).astype(np.float32)        # sums exact in fp32, count a power of two
    np.testing.assert_array_equal(_run_mean(xi, 0, False, False, ws=True),
                                  oracle.reduce_mean(xi.astype(np.float64), 0).astype(np.float32))
    xr = (g.standard_normal((2048, 768)) * 3).astype(np.float32)  # fixed summation order: bit-identical reruns
    np.testing.assert_array_equal(_run_mean(xr, 0, False, False, ws=True), _run_mean(xr, 0, False, False, ws=True))


def test_reduce_mean_bf16_padded_and_exact_integers():
    g = np.random.default_rng(3)
    x = (g.standard_normal((300, 264)) + 1).astype(np.float32)
    xb = _bf16(x)
    for axis in (0, 1):
        y = _run_mean(xb, axis, True, True, ldx=272)
        ref = oracle.reduce_mean(oracle.widen(xb, True), axis)
        got = P.bf16_to_f64(y)
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.maximum(np.abs(ref), 2.0 ** -7) + 1e-5)
        y32 = _run_mean(xb, axis, True, False, ldx=272)
        assert np.max(np.abs(y32 - ref)) <= 1e-5 * 1.5
    xi = g.integers(-8, 9, (128, 64)).astype(np.float32)          # sums exact in fp32, counts powers of two
    np.testing.assert_array_equal(_run_mean(xi, 0, False, False), oracle.reduce_mean(xi.astype(np.float64), 0).astype(np.float32))
    np.testing.assert_array_equal(_run_mean(xi, 1, False, False), oracle.reduce_mean(xi.astype(np.float64), 1).astype(np.float32))


def _run_eltwise(op, a, b, bf16, offset=0):
    n = a.size
    ad = G.dev(np.concatenate([np.zeros(offset, a.dtype), a.ravel()]))
    bd = G.dev(np.concatenate([np.zeros(offset, a.dtype), b.ravel()])) if b is not None else None
    yd = torch.zeros(n + offset, dtype=torch.int16 if bf16 else torch.float32, device="cuda")
    es = 2 if bf16 else 4
    perf.perf_eltwise(op, ad.data_ptr() + es * offset, bd.data_ptr() + es * offset if b is not None else None,
                      yd.data_ptr() + es * offset, n, G.dt(bf16), G.stream())
    torch.cuda.synchronize()
    out = G.host(yd, bf16)
    assert np.all(out[:offset] == 0)
    return out[offset:]


@pytest.mark.parametrize("n", [3072 * 4096, 6 * 14336, 1, 5, 1023, 4096 * 4 + 3])
def test_eltwise_fp32_bit_exact(n):
    g = np.random.default_rng(n % 1000)
    a = (g.standard_normal(n) * 3).astype(np.float32)
    b = (g.standard_normal(n) * 3).astype(np.float32)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    assert np.array_equal(_run_eltwise(perf.PERF_ADD, a, b, False), oracle.round_f32(oracle.eltwise(oracle.ELTWISE_ADD, a64, b64)))
    assert np.array_equal(_run_eltwise(perf.PERF_MUL, a, b, False), oracle.round_f32(oracle.eltwise(oracle.ELTWISE_MUL, a64, b64)))
    r = _run_eltwise(perf.PERF_RELU, a, None, False)
    assert np.array_equal(r, oracle.round_f32(oracle.eltwise(oracle.ELTWISE_RELU, a64)))
    assert not np.any(np.signbit(r))


def test_eltwise_bf16_and_unaligned():
    g = np.random.default_rng(8)
    n = 100003
    a, b = _bf16(g.standard_normal(n) * 2), _bf16(g.standard_normal(n) * 2)
    a64, b64 = oracle.widen(a, True), oracle.widen(b, True)
    for op, oop in ((perf.PERF_ADD, oracle.ELTWISE_ADD), (perf.PERF_MUL, oracle.ELTWISE_MUL)):
        got = _run_eltwise(op, a, b, True)
        want = oracle.round_bf16(oracle.eltwise(oop, a64, b64))
        ulps = np.abs(P.bf16_ordered(got).astype(np.int64) - P.bf16_ordered(want).astype(np.int64))
        assert ulps.max() <= 1 and np.mean(ulps == 0) >= 0.999     # fp32 rounding before the bf16 rounding
    assert np.array_equal(_run_eltwise(perf.PERF_RELU, a, None, True), oracle.round_bf16(oracle.eltwise(oracle.ELTWISE_RELU, a64)))
    af = (g.standard_normal(1000)).astype(np.float32); bf = (g.standard_normal(1000)).astype(np.float32)
    got = _run_eltwise(perf.PERF_ADD, af, bf, False, offset=1)     # 4-byte aligned only: element kernel
    assert np.array_equal(got, af + bf)


def test_stream_probe_copies_and_fills():
    """The measurement aid behind the copy-ceiling study: copy mode must copy bit for bit in every
    launch shape, write mode must fill exactly the requested bytes, read mode must leave dst alone
    (but for its first 16 bytes)."""
    import torch
    n = 1 << 20
    src = torch.randint(0, 255, (n + 64,), dtype=torch.uint8, device="cuda")
    for unroll, threads, grid, policy in ((1, 64, 0, 0), (4, 256, 0, 3), (16, 1024, 7, 1), (8, 512, 300, 2), (2, 128, 0, 3)):
        for nbytes in (n, n - 16 * 37, 16):
            dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
            perf.perf_stream_probe(src.data_ptr(), dst.data_ptr(), nbytes, 0, unroll, threads, grid, policy, G.stream())
            torch.cuda.synchronize()
            assert torch.equal(dst[:nbytes], src[:nbytes]) and not bool(dst[nbytes:].any())
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
    perf.perf_stream_probe(src.data_ptr(), dst.data_ptr(), n, 1, 8, 256, 0, 1, G.stream())
    torch.cuda.synchronize()
    assert not bool(dst[16:].any())
    perf.perf_stream_probe(src.data_ptr(), dst.data_ptr(), n, 2, 8, 256, 0, 2, G.stream())
    torch.cuda.synchronize()
    v = dst[:n].view(torch.int32).view(-1, 4)
    assert bool((v[:, 1] == 1).all()) and bool((v[:, 2] == 2).all()) and not bool(dst[n:].any())


def test_lds_probe_reports_plausible_rates():
    """The LDS probes behind the convolution analysis: the loop runs, the cycle count is written, and
    the rates lie where the hardware allows (one CU: at most 64 banks x 4 bytes x 2 per clock; one MFMA
    32x32x16 takes 32 cycles, so the MFMA + read pattern cannot cost less)."""
    import torch
    cyc = torch.zeros(1, dtype=torch.int64, device="cuda")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    iters = 500
    for waves, nbytes in ((4, 16), (8, 16), (16, 16), (8, 8), (16, 4)):
        cyc.zero_()
        perf.perf_lds_probe(cyc.data_ptr(), sink.data_ptr(), waves, nbytes, 0, iters, G.stream())
        torch.cuda.synchronize()
        rate = waves * iters * 16 * 64 * nbytes / int(cyc.item())
        assert 16.0 < rate <= 512.0, (waves, nbytes, rate)
    for waves in (4, 8):
        cyc.zero_()
        perf.perf_lds_probe(cyc.data_ptr(), sink.data_ptr(), waves, 16, 1, iters, G.stream())
        torch.cuda.synchronize()
        per_mfma = int(cyc.item()) / (iters * 36)
        assert 31.0 < per_mfma < 80.0, (waves, per_mfma)
        cyc.zero_()
        perf.perf_lds_probe(cyc.data_ptr(), sink.data_ptr(), waves, 16, 2, iters, G.stream())
        torch.cuda.synchronize()
        with_valu = int(cyc.item()) / (iters * 36)
        assert per_mfma - 0.5 < with_valu < 80.0, (waves, per_mfma, with_valu)   # extra vector work never makes it faster
    assert float(sink.item()) == 0.0


def test_feed_probe_reports_plausible_rates():
    """The L2 -> CU feed probe: every mode runs, leaves its source untouched, and reports a rate between a trickle
    and what one CU's L1 can take in (64 bytes per clock; the register path with its LDS write can exceed that in
    the probe's own accounting when the window fits the L1, hence the margin)."""
    import torch
    cyc = torch.zeros(1, dtype=torch.int64, device="cuda")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    src = torch.zeros(256 * 65536, dtype=torch.uint8, device="cuda")
    iters = 100
    for shared, span in ((0, 65536), (1, 1 << 20)):
        for waves in (4, 8):
            for mode in range(4):
                cyc.zero_()
                perf.perf_feed_probe(src.data_ptr(), src.numel(), cyc.data_ptr(), sink.data_ptr(), waves, mode, shared, span,
                                     iters, G.stream())
                torch.cuda.synchronize()
                rate = waves * iters * 8192 / int(cyc.item())
                assert 8.0 < rate < 100.0, (shared, span, waves, mode, rate)
    assert float(sink.item()) == 0.0 and not bool(src.any())


def test_copy_any_alignment_and_size():
    """perf_copy (the measured HBM ceiling) must copy bit for bit whatever the alignment of either
    pointer; misaligned cases run grid-wide kernels too (64 MiB in well under a second)."""
    import time
    import torch
    n = 1 << 20
    src = torch.randint(0, 255, (n + 64,), dtype=torch.uint8, device="cuda")
    for so, do, nbytes in ((0, 0, n), (0, 0, n - 5), (1, 0, n - 7), (0, 3, n - 9), (5, 9, n - 11), (7, 7, 3), (2, 1, 40), (0, 8, 16)):
        dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
        perf.perf_copy(src.data_ptr() + so, dst.data_ptr() + do, nbytes, G.stream())
        torch.cuda.synchronize()
        assert torch.equal(dst[do:do + nbytes], src[so:so + nbytes]), (so, do, nbytes)
        assert not bool(dst[:do].any()) and not bool(dst[do + nbytes:].any())
    big = torch.randint(0, 255, ((64 << 20) + 64,), dtype=torch.uint8, device="cuda")
    out = torch.zeros_like(big)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    perf.perf_copy(big.data_ptr() + 1, out.data_ptr() + 2, 64 << 20, G.stream())
    torch.cuda.synchronize()
    assert time.perf_counter() - t0 < 0.5
    assert torch.equal(out[2:2 + (64 << 20)], big[1:1 + (64 << 20)])
