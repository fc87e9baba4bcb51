"""Pins for the softmax oracle: closed forms, invariants and an independent library
routine. None of the expected values below comes from the oracle or from the HIP path."""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import configs


def test_rows_sum_to_one_and_positive():
    x = configs.SoftmaxWorkload(rows=64, cols=1024).make()["x"]
    y = oracle.softmax(x)
    assert np.all(y > 0)
    assert np.max(np.abs(y.sum(axis=1) - 1.0)) < 1e-12


def test_shift_invariance():
    x = configs.SoftmaxWorkload(rows=16, cols=333).make()["x"].astype(np.float64)
    y0 = oracle.softmax(x)
    y1 = oracle.softmax(x + 37.25)
    assert np.max(np.abs(y0 - y1) / y0) < 1e-12


def test_constant_row_is_uniform():
    y = oracle.softmax(np.full((3, 1024), -7.5))
    assert np.array_equal(y, np.full((3, 1024), 2.0 ** -10))


def test_two_element_row_is_logistic():
    for a, b in [(0.3, -1.2), (5.0, 5.5), (-40.0, 2.0)]:
        y = oracle.softmax(np.array([[a, b]]))
        assert y[0, 0] == pytest.approx(1.0 / (1.0 + math.exp(b - a)), rel=1e-14)
        assert y[0, 1] == pytest.approx(1.0 / (1.0 + math.exp(a - b)), rel=1e-14)


def test_log_row_gives_proportions():
    y = oracle.softmax(np.log(np.array([[1.0, 2.0, 3.0, 4.0]])))
    assert np.allclose(y, [[0.1, 0.2, 0.3, 0.4]], rtol=0, atol=1e-15)


def test_dominant_entry_saturates_in_fp32():
    x = np.zeros((1, 512))
    x[0, 77] = 104.0
    y32 = oracle.round_f32(oracle.softmax(x))
    expect = np.zeros((1, 512), dtype=np.float32)
    expect[0, 77] = 1.0
    assert np.array_equal(y32, expect)
    assert not np.isnan(y32).any()


def test_scale_multiplies_logits():
    x = configs.SoftmaxWorkload(rows=8, cols=100).make()["x"].astype(np.float64)
    assert np.allclose(oracle.softmax(x, scale=0.125), oracle.softmax(x * 0.125), rtol=1e-14, atol=0)
    # a negative scale reverses the order: the smallest logit gets the largest probability
    y = oracle.softmax(x, scale=-1.0)
    assert np.array_equal(y.argmax(axis=1), x.argmin(axis=1))


def test_monotone_so_argmax_matches_input():
    x = configs.CONFIG1.make()["x"]
    y = oracle.softmax(x)
    assert np.array_equal(y.argmax(axis=1), x.argmax(axis=1))
    order_x = np.argsort(x[0], kind="stable")
    assert np.all(np.diff(y[0][order_x]) >= 0)


def test_single_column():
    assert np.array_equal(oracle.softmax(np.array([[3.0], [-2.0]])), np.ones((2, 1)))


def test_against_torch_float64():
    x = configs.CONFIG1.make()["x"]
    ref = torch.softmax(torch.from_numpy(x).double(), dim=-1).numpy()
    y = oracle.softmax(x)
    assert np.max(np.abs(y - ref) / ref) < 1e-13
    ref8 = torch.softmax(torch.from_numpy(x).double() * 0.125, dim=-1).numpy()
    assert np.max(np.abs(oracle.softmax(x, 0.125) - ref8) / ref8) < 1e-13
