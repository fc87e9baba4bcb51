"""GPU parity: perf_gemm (MFMA and general kernels) against the CPU oracle.
Tolerance for bf16-input / fp32-accumulate results: max |C^-C| / max(|C|, rms(C)) <= 2e-2,
plus the accumulation-order-independent bound |C^-C| <= K 2^-23 sum_k|a||b|. Exact-integer
problems must match bit for bit."""
import numpy as np
import pytest

import oracle
from workloads import configs, rng
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def _bits(a):
    return rng.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _check(wl, alpha=1.0, c_bf16=False, batch=1, **kw):
    d = wl.make()
    a, b = d["a_bf16"], d["b_bf16"]
    if batch > 1:
        a = np.stack([np.roll(a, i, axis=0) for i in range(batch)])
        b = np.stack([np.roll(b, -i, axis=1) for i in range(batch)])
    c = G.run_gemm(a, b, wl.M, wl.N, wl.K, alpha=alpha, batch=batch, c_bf16=c_bf16, **kw)
    ad, bd = oracle.widen(a, bf16=True), oracle.widen(b, bf16=True)
    ref = oracle.gemm(ad, bd, wl.M, wl.N, wl.K, b_col=True, alpha=float(np.float32(alpha)), batch=batch)
    ref = ref.reshape(batch, wl.M, wl.N)
    for i in range(batch):
        ai = ad.reshape(batch, -1)[i]
        bi = bd.reshape(batch, -1)[i]
        s = abs(float(np.float32(alpha))) * oracle.gemm_absdot(ai, bi, wl.M, wl.N, wl.K, b_col=True)
        ci = P.bf16_to_f64(c[i]) if c_bf16 else c[i]
        P.assert_contraction_close(ci, ref[i], s, wl.K, out_bf16=c_bf16)


@pytest.mark.parametrize("M,N,K", [
    (256, 256, 64), (128, 128, 128), (256, 512, 256), (300, 200, 192), (1, 1, 64), (257, 129, 128),
    (64, 640, 64), (33, 7, 512), (768, 1024, 1024), (512, 512, 64),
])
def test_mfma_path_shapes_and_tails(M, N, K):
    _check(configs.GemmWorkload(M=M, N=N, K=K))


def test_mfma_large_tile_path_with_tails():
    # enough 256x256 tiles to select the 4x4-wave-tile kernel, with ragged M and N
    _check(configs.GemmWorkload(M=4096 - 37, N=4096 + 19, K=128))


def test_alpha_bf16_output_batched_and_padded_ld():
    _check(configs.GemmWorkload(M=160, N=96, K=128), alpha=0.125)
    _check(configs.GemmWorkload(M=160, N=96, K=128), c_bf16=True)
    _check(configs.GemmWorkload(M=130, N=70, K=64), alpha=0.125, batch=5)
    wl = configs.GemmWorkload(M=96, N=80, K=64)
    d = wl.make()
    a = np.zeros((96, 72), np.uint16); a[:, :64] = d["a_bf16"]
    b = np.zeros((80, 88), np.uint16); b[:, :64] = d["b_bf16"]
    c = G.run_gemm(a, b, 96, 80, 64, lda=72, ldb=88, ldc=84)[0]
    ref = oracle.gemm(oracle.widen(d["a_bf16"], True), oracle.widen(d["b_bf16"], True), 96, 80, 64, b_col=True)
    s = oracle.gemm_absdot(oracle.widen(d["a_bf16"], True), oracle.widen(d["b_bf16"], True), 96, 80, 64, b_col=True)
    P.assert_contraction_close(c, ref, s, 64)


def test_mid_tile_kernels():
    # 128x128 tiles are chosen between 192 such tiles and 256 tiles of 256x256; smaller problems get 64x64 tiles
    _check(configs.GemmWorkload(M=1792, N=1800, K=64))      # K-step-32 loop, 128x128 tiles, ragged N
    _check(configs.GemmWorkload(M=1792, N=1792, K=512))     # 128x128 tiles, long reduction
    _check(configs.GemmWorkload(M=1792, N=1792, K=512), tile=128, kstep=64)


def test_k64_loop_tails_alpha_bf16_batched_and_odd_ldc():
    # the K-step-64 loop (16x16x32 MFMAs, lane-exchange epilogue, bf16 C staged through LDS); the
    # library picks it for 256x256 tiles with K a multiple of 64 and >= 512, the smaller tiles are named
    _check(configs.GemmWorkload(M=300, N=200, K=576), tile=128, kstep=64)      # ragged, odd step count
    _check(configs.GemmWorkload(M=256, N=384, K=512), alpha=0.125, tile=128, kstep=64)  # full tiles, vector epilogue, alpha
    _check(configs.GemmWorkload(M=256, N=256, K=512), c_bf16=True, tile=128, kstep=64)  # bf16 epilogue through LDS
    _check(configs.GemmWorkload(M=256, N=256, K=512), c_bf16=True, tile=64, kstep=64)
    _check(configs.GemmWorkload(M=512, N=256, K=128), c_bf16=True, tile=256, kstep=64)
    _check(configs.GemmWorkload(M=130, N=70, K=512), alpha=-2.0, batch=3, c_bf16=True, tile=128, kstep=64)
    _check(configs.GemmWorkload(M=130, N=70, K=512), alpha=-2.0, batch=3, c_bf16=True, tile=64, kstep=64)
    _check(configs.GemmWorkload(M=512, N=512, K=512), batch=64)                # 256 tiles of 256x256: the large-tile kernel
    _check(configs.GemmWorkload(M=512, N=512, K=512), batch=64, c_bf16=True)
    _check(configs.GemmWorkload(M=2048 + 40, N=2048 - 24, K=640))              # large-tile kernel with ragged edges
    wl = configs.GemmWorkload(M=256, N=256, K=512)
    d = wl.make()
    c = G.run_gemm(d["a_bf16"], d["b_bf16"], 256, 256, 512, ldc=258, tile=128, kstep=64)[0]  # ldc not a multiple of 4: scalar epilogue
    ad, bd = oracle.widen(d["a_bf16"], True), oracle.widen(d["b_bf16"], True)
    ref = oracle.gemm(ad, bd, 256, 256, 512, b_col=True)
    P.assert_contraction_close(c, ref, oracle.gemm_absdot(ad, bd, 256, 256, 512, b_col=True), 512)

@pytest.mark.gpu
def test_k64_loop_with_32x32_mfma():
    """The K-step-64 loop of the 256x256 tile built on the 32x32x16 MFMA: ragged edges, several k-steps, alpha, batch, bf16 C."""
    _check(configs.GemmWorkload(M=512, N=256, K=128), tile=256, kstep=65)
    _check(configs.GemmWorkload(M=300, N=520, K=576), tile=256, kstep=65, alpha=0.25)
    _check(configs.GemmWorkload(M=258, N=130, K=64), tile=256, kstep=65, batch=2, c_bf16=True)
    _check(configs.GemmWorkload(M=1024, N=768, K=1024), tile=256, kstep=65, c_bf16=True)



def test_deep_ring_loop():
    # K-step-32 loop with the ring filling the LDS (16 stages of a 64x64 tile, 8 of a 128x128 one):
    # reductions shorter than, equal to and longer than the ring, ragged tiles, batches, bf16 C
    for tile in (64, 128):
        _check(configs.GemmWorkload(M=100, N=70, K=64), tile=tile, kstep=33)
        _check(configs.GemmWorkload(M=192, N=130, K=512), tile=tile, kstep=33, alpha=0.5)
        _check(configs.GemmWorkload(M=130, N=260, K=1056), tile=tile, kstep=33, batch=2, c_bf16=True)
    _check(configs.GemmWorkload(M=512, N=512, K=2048))      # one round of 64x64 tiles, long reduction: the library's own choice


@pytest.mark.parametrize("a_col,b_col", [(False, False), (True, False), (True, True), (False, True)])
@pytest.mark.parametrize("M,N,K", [(5, 7, 3), (65, 63, 17), (100, 130, 65)])
def test_general_kernel_layouts_exact_integers(a_col, b_col, M, N, K):
    g = np.random.default_rng(M + N + K)
    a = g.integers(-8, 9, (M, K)).astype(np.float32)
    b = g.integers(-8, 9, (K, N)).astype(np.float32)
    a_st = a.T.copy() if a_col else a
    b_st = b.T.copy() if b_col else b
    ref = oracle.gemm(a_st, b_st, M, N, K, a_col=a_col, b_col=b_col, alpha=0.5)
    c16 = G.run_gemm(_bits(a_st), _bits(b_st), M, N, K, a_col=a_col, b_col=b_col, alpha=0.5)[0]
    c32 = G.run_gemm(a_st, b_st, M, N, K, a_col=a_col, b_col=b_col, alpha=0.5, ab_bf16=False)[0]
    assert np.array_equal(c16.astype(np.float64), ref) and np.array_equal(c32.astype(np.float64), ref)


def test_mfma_exact_integers_identity_permutation_ones():
    g = np.random.default_rng(3)
    M, N, K = 200, 136, 192
    a = g.integers(-8, 9, (M, K)).astype(np.float32)
    bs = g.integers(-8, 9, (N, K)).astype(np.float32)           # column-major storage of B
    ref = oracle.gemm(a, bs, M, N, K, b_col=True)
    assert np.array_equal(G.run_gemm(_bits(a), _bits(bs), M, N, K)[0].astype(np.float64), ref)
    n = 128
    a = rng.bf16_bits_to_f32(configs.GemmWorkload(M=n, N=n, K=n).make()["a_bf16"])
    eye = np.eye(n, dtype=np.float32)
    assert np.array_equal(G.run_gemm(_bits(a), _bits(eye), n, n, n)[0], a)            # B = I
    assert np.array_equal(G.run_gemm(_bits(eye), _bits(a), n, n, n)[0], a.T)          # A = I: C = B = storage^T
    # cyclic shift: B[k][n] = [k == (n+1) mod K]; stored column-major => bs[n][k]
    bs = np.zeros((n, n), np.float32)
    for col in range(n):
        bs[col, (col + 1) % n] = 1.0
    assert np.array_equal(G.run_gemm(_bits(a), _bits(bs), n, n, n)[0], np.roll(a, -1, axis=1))
    ones = G.run_gemm(_bits(np.ones((70, 320))), _bits(np.ones((90, 320))), 70, 90, 320)[0]
    assert np.array_equal(ones, np.full((70, 90), 320.0, np.float32))


@pytest.mark.parametrize("tile,kstep", [(0, 0), (256, 65)])
def test_config3_full_size_sampled_rows(tile, kstep):
    """4096^3 in the benchmark's launch configuration (and with the 32x32x16 variant of its main
    loop); 48 sampled rows of C (all columns) are recomputed by the oracle, and the whole C is
    checked against row/column sums."""
    wl = configs.CONFIG3
    d = wl.make()
    c = G.run_gemm(d["a_bf16"], d["b_bf16"], wl.M, wl.N, wl.K, tile=tile, kstep=kstep)[0]
    rows = np.unique(np.concatenate([np.arange(0, wl.M, 89), [255, 256, 4095]]))
    a_s = oracle.widen(d["a_bf16"][rows], True)
    bd = oracle.widen(d["b_bf16"], True)
    ref = oracle.gemm(a_s, bd, len(rows), wl.N, wl.K, b_col=True)
    s = oracle.gemm_absdot(a_s, bd, len(rows), wl.N, wl.K, b_col=True)
    P.assert_contraction_close(c[rows], ref, s, wl.K)
    # property over every entry: C @ 1 = A @ (B @ 1), in float64 (tolerance: fp32 accumulation
    # error of one entry, <= K 2^-23 sum|a||b| <= K^2 2^-23, times sqrt(N) for the sum)
    af = oracle.widen(d["a_bf16"], True)
    rowsum_ref = af @ bd.sum(axis=0)
    assert np.max(np.abs(c.astype(np.float64).sum(axis=1) - rowsum_ref)) < 1.0


@pytest.mark.parametrize("c_bf16", [False, True])
def test_config3_full_size_every_entry_exact_integers(c_bf16):
    """4096^3 in the benchmark's launch configuration with small-integer operands (|v| <= 8): every
    product and every partial sum is an integer below 2^24, exact in fp32 whatever the order, so
    all 16.7M entries of C must equal the exact product bit for bit. The exact product is a float64
    matmul on the host (exact for the same reason), tied to the oracle on sampled rows. With bf16 C
    the expected bits are the oracle's single rounding of the exact value."""
    wl = configs.CONFIG3
    g = np.random.default_rng(303)
    a = g.integers(-8, 9, (wl.M, wl.K)).astype(np.float32)
    bs = g.integers(-8, 9, (wl.N, wl.K)).astype(np.float32)      # column-major storage of B
    exact = a.astype(np.float64) @ bs.astype(np.float64).T
    rows = np.array([0, 255, 256, 1777, 4095])
    assert np.array_equal(oracle.gemm(a[rows].astype(np.float64), bs.astype(np.float64), len(rows), wl.N, wl.K, b_col=True),
                          exact[rows])
    c = G.run_gemm(_bits(a), _bits(bs), wl.M, wl.N, wl.K, c_bf16=c_bf16)[0]
    if c_bf16:
        assert np.array_equal(c, oracle.round_bf16(exact))
    else:
        assert np.array_equal(c.astype(np.float64), exact)


def test_config4_attention_scores_then_softmax():
    """Q K^T / 8 for 512 (batch x head) matrices, then row softmax of the 262144 x 512
    scores: all batches on the GPU; three batches recomputed by the oracle."""
    import torch
    import paper_2511_03586_amd as perf
    wl = configs.CONFIG4
    d = wl.make()
    qd, kd = G.dev(d["q_bf16"]), G.dev(d["k_bf16"])
    S, D, B = wl.seq, wl.d, wl.batch
    sd = torch.empty(B * S * S, dtype=torch.float32, device="cuda")
    pd = torch.empty_like(sd)
    perf.perf_gemm(qd.data_ptr(), kd.data_ptr(), sd.data_ptr(), S, S, D, perf.PERF_ROW_MAJOR, D,
                   perf.PERF_COL_MAJOR, D, S, B, S * D, S * D, S * S, wl.alpha, perf.PERF_BF16, perf.PERF_F32,
                   G.stream())
    perf.perf_softmax(sd.data_ptr(), pd.data_ptr(), B * S, S, S, S, perf.PERF_F32, perf.PERF_F32, 1.0, G.stream())
    torch.cuda.synchronize()
    assert float((pd.view(B * S, S).double().sum(dim=1) - 1.0).abs().max()) < 1e-5
    for b in (0, 257, 511):
        q, k = oracle.widen(d["q_bf16"][b], True), oracle.widen(d["k_bf16"][b], True)
        s_ref = oracle.gemm(q, k, S, S, D, b_col=True, alpha=wl.alpha)
        absdot = wl.alpha * oracle.gemm_absdot(q, k, S, S, D, b_col=True)
        s_gpu = sd.view(B, S, S)[b].cpu().numpy()
        P.assert_contraction_close(s_gpu, s_ref, absdot, D)
        p_gpu = pd.view(B, S, S)[b].cpu().numpy()
        P.assert_softmax_close(p_gpu, oracle.softmax(s_ref))
        # argmax exact on rows the oracle can decide (top-two scores more than 1e-5 apart)
        top2 = np.sort(s_ref, axis=1)[:, -2:]
        decidable = (top2[:, 1] - top2[:, 0]) > 1e-5
        assert np.array_equal(p_gpu.argmax(axis=1)[decidable], s_ref.argmax(axis=1)[decidable])


def test_deterministic():
    d = configs.GemmWorkload(M=512, N=512, K=512).make()
    c0 = G.run_gemm(d["a_bf16"], d["b_bf16"], 512, 512, 512)
    c1 = G.run_gemm(d["a_bf16"], d["b_bf16"], 512, 512, 512)
    assert np.array_equal(c0, c1)
