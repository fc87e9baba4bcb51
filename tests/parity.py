"""Tolerance checks used by the GPU parity tests. Every tolerance is written out here."""
import numpy as np

from workloads import rng


def bf16_ordered(bits: np.ndarray) -> np.ndarray:
    """Map bf16 bit patterns to integers whose order and spacing follow the real line,
    so |a - b| counts bf16 units in the last place between two values."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def softmax_max_rel_err(y_gpu: np.ndarray, y_ref: np.ndarray):
    """max |y_gpu - y| / y over entries with y >= 1e-30; max |y_gpu - y| below that."""
    y_gpu = y_gpu.astype(np.float64)
    big = y_ref >= 1e-30
    rel = np.max(np.abs(y_gpu[big] - y_ref[big]) / y_ref[big]) if big.any() else 0.0
    small = np.max(np.abs(y_gpu[~big] - y_ref[~big])) if (~big).any() else 0.0
    return rel, small


def assert_softmax_close(y_gpu, y_ref, tol=1e-5):
    rel, small = softmax_max_rel_err(y_gpu, y_ref)
    assert rel <= tol, f"softmax max relative error {rel:.3e} > {tol}"
    assert small <= 1e-35, f"softmax absolute error below the floor {small:.3e}"


def assert_argmax_exact(y_gpu, x_scaled_ref):
    """argmax per row must equal the oracle's; a row whose two largest logits are equal
    may pick either (lowest-index convention otherwise)."""
    am = y_gpu.argmax(axis=1)
    ref = x_scaled_ref.argmax(axis=1)
    bad = np.nonzero(am != ref)[0]
    for r in bad:
        assert x_scaled_ref[r, am[r]] == x_scaled_ref[r, ref[r]], f"row {r}: argmax {am[r]} != {ref[r]}"


def contraction_errors(c_gpu, c_ref, absdot=None):
    """(contract gate, sharp gate) for bf16-input fp32-accumulate contractions:
    max |C^ - C| / max(|C|, rms(C))   and   max |C^ - C| / sum_k |a||b|."""
    c_gpu = c_gpu.astype(np.float64)
    diff = np.abs(c_gpu - c_ref)
    rms = np.sqrt(np.mean(c_ref ** 2))
    gate = np.max(diff / np.maximum(np.abs(c_ref), max(rms, 1e-300)))
    sharp = np.max(diff / np.maximum(absdot, 1e-300)) if absdot is not None else None
    return gate, sharp


def assert_contraction_close(c_gpu, c_ref, absdot, K, out_bf16=False):
    """Contract gate 2e-2; sharp gate: any fp32 accumulation order obeys
    |err| <= K * 2^-23 * sum|a||b| (+ one bf16 rounding of the result, 2^-8 |C|, if the
    output is bf16)."""
    gate, _ = contraction_errors(c_gpu, c_ref, absdot)
    assert gate <= 2e-2, f"relative error (rms floor) {gate:.3e} > 2e-2"
    bound = K * 2.0 ** -23 * absdot + 2.0 ** -24 * np.abs(c_ref)
    if out_bf16:
        bound = bound + 2.0 ** -8 * np.abs(c_ref) + 2.0 ** -133
    worst = np.max(np.abs(c_gpu.astype(np.float64) - c_ref) - bound)
    assert worst <= 0, f"error exceeds the accumulation-order-independent bound by {worst:.3e}"
    return gate


def bf16_to_f64(bits):
    return rng.bf16_bits_to_f32(bits).astype(np.float64)
