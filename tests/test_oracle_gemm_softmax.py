"""Pins for the oracle's fused score-GEMM + softmax composition ("bmm" then "softmax" rows of the
paper's operator table, Section 4.3): closed forms and a second opinion that shares no code
with it (numpy matmul + the textbook formula)."""
import numpy as np

import oracle


def test_two_column_logistic_closed_form():
    # M=1, N=2, K=1: scores (alpha*t*1, alpha*t*0) -> P = (1/(1+e^{-alpha t}), 1/(1+e^{alpha t}))
    for t, alpha in ((0.0, 1.0), (2.0, 0.5), (-3.0, 1.0), (1.5, -2.0)):
        p = oracle.gemm_softmax(np.array([t]), np.array([1.0, 0.0]), 1, 2, 1, alpha=alpha)[0, 0]
        z = alpha * t
        np.testing.assert_allclose(p, [1 / (1 + np.exp(-z)), 1 / (1 + np.exp(z))], rtol=1e-15)


def test_log_rows_give_prescribed_probabilities():
    # A = I (K = M), B[n][k] = ln(w[k][n]): scores ln w -> each row is w / sum(w); pins the B^T convention
    w = np.array([[1.0, 2.0, 3.0, 4.0], [5.0, 1.0, 1.0, 3.0], [2.0, 2.0, 2.0, 2.0]])      # [k][n]
    b = np.log(w).T.copy()                                                                 # N rows of K
    p = oracle.gemm_softmax(np.eye(3), b, 3, 4, 3)[0]
    np.testing.assert_allclose(p, w / w.sum(1, keepdims=True), rtol=1e-14)


def test_rows_sum_to_one_and_batches_are_independent():
    g = np.random.default_rng(5)
    a = g.standard_normal((3, 7, 16))
    b = g.standard_normal((3, 9, 16))
    p = oracle.gemm_softmax(a, b, 7, 9, 16, alpha=0.25, batch=3)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-13)
    for i in range(3):
        np.testing.assert_array_equal(p[i], oracle.gemm_softmax(a[i], b[i], 7, 9, 16, alpha=0.25)[0])


def test_against_numpy_formula():
    g = np.random.default_rng(11)
    a = g.standard_normal((2, 33, 24))
    b = g.standard_normal((2, 17, 24))
    s = -0.75 * np.einsum("bmk,bnk->bmn", a, b)
    e = np.exp(s - s.max(-1, keepdims=True))
    np.testing.assert_allclose(oracle.gemm_softmax(a, b, 33, 17, 24, alpha=-0.75, batch=2),
                               e / e.sum(-1, keepdims=True), rtol=1e-12)
