"""Pins for the GEMM oracle: brute force on tiny exact-integer problems, identity,
a non-involutive permutation, all-ones, numpy float64."""
import numpy as np
import pytest

import oracle
from workloads import configs, rng


def _brute(a_rm, b_rm, alpha=1.0):
    """Pure-Python triple loop, n-outer / m-inner / k descending: a different nest from
    the oracle's. Integer data keeps every sum exact, so order does not matter."""
    M, K = a_rm.shape
    N = b_rm.shape[1]
    c = np.zeros((M, N))
    for n in range(N):
        for m in range(M):
            s = 0.0
            for k in range(K - 1, -1, -1):
                s += float(a_rm[m, k]) * float(b_rm[k, n])
            c[m, n] = alpha * s
    return c


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (17, 5, 3), (5, 17, 33), (33, 2, 17), (9, 7, 20)])
@pytest.mark.parametrize("a_col,b_col", [(False, False), (False, True), (True, False), (True, True)])
def test_brute_force_exact_integers(M, N, K, a_col, b_col):
    g = np.random.default_rng(M * 1000 + N * 10 + K)
    a = g.integers(-8, 9, (M, K)).astype(np.float64)     # logical A[m,k]
    b = g.integers(-8, 9, (K, N)).astype(np.float64)     # logical B[k,n]
    a_store = a.T.copy() if a_col else a                 # col-major: storage index k*lda+m
    b_store = b.T.copy() if b_col else b                 # col-major: storage index n*ldb+k
    c = oracle.gemm(a_store, b_store, M, N, K, a_col=a_col, b_col=b_col, alpha=0.5)
    assert np.array_equal(c, _brute(a, b, 0.5))


def test_identity_b_returns_a_and_identity_a_returns_b():
    g = np.random.default_rng(1)
    n = 37
    a = g.standard_normal((n, n))
    assert np.array_equal(oracle.gemm(a, np.eye(n), n, n, n, b_col=True), a)
    # A = I, B column-major storage bs[n][k] = B[k][n]  =>  C = B = bs^T
    bs = g.standard_normal((n, n))
    assert np.array_equal(oracle.gemm(np.eye(n), bs, n, n, n, b_col=True), bs.T)
    assert np.array_equal(oracle.gemm(np.eye(n), bs, n, n, n, b_col=False), bs)


def test_cyclic_shift_permutation_rotates_columns():
    # B[k][n] = 1 iff k == (n+1) mod K  =>  C[m][n] = A[m][(n+1) mod K]: columns rotate
    # left. P != P^T, so reading B with the wrong layout rotates the other way.
    g = np.random.default_rng(2)
    M, K = 11, 13
    a = g.standard_normal((M, K))
    b = np.zeros((K, K))
    for n in range(K):
        b[(n + 1) % K, n] = 1.0
    expect = np.roll(a, -1, axis=1)
    assert np.array_equal(oracle.gemm(a, b, M, K, K, b_col=False), expect)
    assert np.array_equal(oracle.gemm(a, b.T.copy(), M, K, K, b_col=True), expect)
    assert not np.array_equal(oracle.gemm(a, b, M, K, K, b_col=True), expect)


def test_all_ones_counts_k():
    M, N, K = 6, 9, 257
    c = oracle.gemm(np.ones((M, K)), np.ones((N, K)), M, N, K, b_col=True)
    assert np.array_equal(c, np.full((M, N), float(K)))


def test_batched_strides_and_alpha():
    g = np.random.default_rng(4)
    B, M, N, K = 5, 7, 6, 9
    a = g.integers(-4, 5, (B, M, K)).astype(np.float64)
    bs = g.integers(-4, 5, (B, N, K)).astype(np.float64)          # column-major storage
    c = oracle.gemm(a, bs, M, N, K, b_col=True, alpha=0.125, batch=B)
    for i in range(B):
        assert np.array_equal(c[i], 0.125 * (a[i] @ bs[i].T))


def test_against_numpy_float64_on_workload_recipe():
    wl = configs.GemmWorkload(M=96, N=80, K=512)
    d = wl.make()
    a = rng.bf16_bits_to_f32(d["a_bf16"]).astype(np.float64)
    b = rng.bf16_bits_to_f32(d["b_bf16"]).astype(np.float64)
    c = oracle.gemm(a, b, wl.M, wl.N, wl.K, b_col=True)
    ref = a @ b.T
    s = oracle.gemm_absdot(a, b, wl.M, wl.N, wl.K, b_col=True)
    assert np.allclose(s, np.abs(a) @ np.abs(b.T), rtol=1e-13)
    assert np.max(np.abs(c - ref) / s) < 1e-14
    # inputs are U[-1,1] rounded to bf16: |a| <= 1 and not degenerate
    assert np.abs(a).max() <= 1.0 and 0.3 < a.var() < 0.36


def test_attention_scores_closed_forms():
    # K = 0 -> all scores 0 -> uniform probabilities 1/seq exactly
    seq, d = 64, 16
    q = np.random.default_rng(7).standard_normal((2, seq, d))
    s = oracle.gemm(q, np.zeros((2, seq, d)), seq, seq, d, b_col=True, alpha=0.125, batch=2)
    p = oracle.softmax(s.reshape(-1, seq))
    assert np.array_equal(p, np.full((2 * seq, seq), 1.0 / seq))
    # Q = K = c * (rows of an orthonormal basis): S = alpha c^2 I, so
    # P_ii = e^{alpha c^2} / (e^{alpha c^2} + seq - 1), off-diagonal 1 / (same denominator)
    n = 16
    qmat, _ = np.linalg.qr(np.random.default_rng(8).standard_normal((n, n)))
    c = 6.0
    s = oracle.gemm(c * qmat, c * qmat, n, n, n, b_col=True, alpha=0.125)
    p = oracle.softmax(s)
    e = np.exp(0.125 * c * c)
    assert np.allclose(np.diag(p), e / (e + n - 1), rtol=1e-12)
    assert np.allclose(p[~np.eye(n, dtype=bool)], 1.0 / (e + n - 1), rtol=1e-11)
