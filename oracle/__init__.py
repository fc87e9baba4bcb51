"""ctypes front end of the CPU oracle (``oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``; never by the product package. It shares no
code with the HIP path. All results are float64; ``round_f32`` / ``round_bf16`` apply
the single final rounding to an output type.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (no fast-math) into liboracle.so next to it."""
    src = os.path.join(_HERE, "oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-fno-fast-math", "-o", _SO, src, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        i64, dbl, ptr, cint = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.oracle_max_threads.restype = cint
        lib.oracle_set_threads.argtypes = [cint]
        lib.oracle_softmax.argtypes = [ptr, ptr, i64, i64, i64, i64, dbl]
        lib.oracle_layernorm.argtypes = [ptr, ptr, ptr, ptr, ptr, ptr, i64, i64, i64, i64, dbl]
        lib.oracle_gemm.argtypes = [ptr, ptr, ptr, i64, i64, i64, cint, i64, cint, i64, i64,
                                    i64, i64, i64, i64, dbl]
        lib.oracle_gemm_absdot.argtypes = [ptr, ptr, ptr, i64, i64, i64, cint, i64, cint, i64, i64]
        lib.oracle_conv2d.argtypes = [ptr, ptr, ptr, ptr] + [i64] * 11
        lib.oracle_rmsnorm.argtypes = [ptr, ptr, ptr, ptr, i64, i64, dbl]
        lib.oracle_reduce_mean.argtypes = [ptr, ptr, i64, i64, cint]
        lib.oracle_batchnorm.argtypes = [ptr, ptr, ptr, ptr, ptr, ptr, i64, i64, i64, dbl]
        lib.oracle_eltwise.argtypes = [cint, ptr, ptr, ptr, i64]
        lib.oracle_round_f32.argtypes = [ptr, ptr, i64]
        lib.oracle_round_bf16.argtypes = [ptr, ptr, i64]
        for f in ("oracle_set_threads", "oracle_softmax", "oracle_layernorm", "oracle_gemm",
                  "oracle_gemm_absdot", "oracle_conv2d", "oracle_round_f32", "oracle_round_bf16",
                  "oracle_rmsnorm", "oracle_reduce_mean", "oracle_eltwise", "oracle_batchnorm"):
            getattr(lib, f).restype = None
        _lib = lib
    return _lib


def max_threads() -> int:
    return _load().oracle_max_threads()


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def widen(a, bf16: bool = False) -> np.ndarray:
    """Exact widening to a C-contiguous float64 array. ``bf16=True``: ``a`` holds bf16
    bit patterns (uint16), whose value is the fp32 number with those top 16 bits."""
    a = np.asarray(a)
    if bf16:
        assert a.dtype == np.uint16
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def softmax(x: np.ndarray, scale: float = 1.0) -> np.ndarray:
    """Row softmax of scale*x over the last axis of a 2-D float64 array."""
    x = widen(x)
    rows, cols = x.shape
    y = np.empty_like(x)
    _load().oracle_softmax(_p(x), _p(y), rows, cols, cols, cols, float(scale))
    return y


def layernorm(x, gamma, beta, eps: float):
    """Returns (y, mean, rstd), all float64; x is 2-D, gamma/beta 1-D of length cols."""
    x, gamma, beta = widen(x), widen(gamma), widen(beta)
    rows, cols = x.shape
    assert gamma.shape == (cols,) and beta.shape == (cols,)
    y = np.empty_like(x)
    mean = np.empty(rows, dtype=np.float64)
    rstd = np.empty(rows, dtype=np.float64)
    _load().oracle_layernorm(_p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(rstd),
                             rows, cols, cols, cols, float(eps))
    return y, mean, rstd


def rmsnorm(x, gamma, eps: float):
    """Returns (y, rrms), float64; x is 2-D, gamma 1-D of length cols."""
    x, gamma = widen(x), widen(gamma)
    rows, cols = x.shape
    assert gamma.shape == (cols,)
    y = np.empty_like(x)
    r = np.empty(rows, dtype=np.float64)
    _load().oracle_rmsnorm(_p(x), _p(gamma), _p(y), _p(r), rows, cols, float(eps))
    return y, r


def batchnorm(x, gamma, beta, eps: float):
    """x: [N, C, H, W] (or [N, C, HW]) float64; batch statistics per channel. Returns (y, mean, rstd)."""
    x, gamma, beta = widen(x), widen(gamma), widen(beta)
    N, C = x.shape[0], x.shape[1]
    HW = int(np.prod(x.shape[2:]))
    assert gamma.shape == (C,) and beta.shape == (C,)
    y = np.empty_like(x)
    m = np.empty(C, dtype=np.float64)
    r = np.empty(C, dtype=np.float64)
    _load().oracle_batchnorm(_p(x), _p(gamma), _p(beta), _p(y), _p(m), _p(r), N, C, HW, float(eps))
    return y, m, r


def reduce_mean(x, axis: int):
    """Mean of a 2-D float64 array along ``axis`` (0 or 1)."""
    x = widen(x)
    rows, cols = x.shape
    y = np.empty(rows if axis == 1 else cols, dtype=np.float64)
    _load().oracle_reduce_mean(_p(x), _p(y), rows, cols, int(axis))
    return y


ELTWISE_ADD, ELTWISE_MUL, ELTWISE_RELU = 0, 1, 2


def eltwise(op: int, a, b=None):
    """Element-wise add / mul / relu of float64 arrays (b unused for relu)."""
    a = widen(a)
    b = widen(b) if b is not None else a
    assert a.shape == b.shape
    y = np.empty_like(a)
    _load().oracle_eltwise(int(op), _p(a.ravel()), _p(b.ravel()), _p(y.reshape(-1)), a.size)
    return y


def gemm(a, b, M, N, K, a_col=False, b_col=False, alpha=1.0, batch=1, lda=None, ldb=None):
    """C[b] = alpha * A[b] @ B[b]. ``a`` and ``b`` are flat (or any-shape contiguous)
    float64 storage; the layout flags say how (m,k) / (k,n) map into it:
    row-major A[m*lda+k], col-major A[k*lda+m]; row-major B[k*ldb+n], col-major B[n*ldb+k].
    Batches are densely packed. Returns float64 [batch, M, N] (or [M, N] if batch == 1)."""
    a, b = widen(a).ravel(), widen(b).ravel()
    lda = lda if lda is not None else (M if a_col else K)
    ldb = ldb if ldb is not None else (K if b_col else N)
    sa = lda * (K if a_col else M)
    sb = ldb * (N if b_col else K)
    assert a.size >= batch * sa and b.size >= batch * sb
    c = np.empty((batch, M, N), dtype=np.float64)
    _load().oracle_gemm(_p(a), _p(b), _p(c), M, N, K, int(a_col), lda, int(b_col), ldb, N,
                        batch, sa, sb, M * N, float(alpha))
    return c[0] if batch == 1 else c


def gemm_softmax(a, b, M, N, K, alpha=1.0, batch=1):
    """P[b] = softmax_rows(alpha * A[b] @ B[b]^T): the "bmm" then "softmax" pair of the operator
    table (Section 4.3 of the paper) as the plain composition of the two definitions above.
    A is row-major [M,K], B holds N rows of K (column-major K x N), batches densely packed.
    Returns float64 [batch, M, N]."""
    s = gemm(a, b, M, N, K, a_col=False, b_col=True, alpha=alpha, batch=batch)
    return softmax(np.ascontiguousarray(s).reshape(batch * M, N), 1.0).reshape(batch, M, N)


def gemm_absdot(a, b, M, N, K, a_col=False, b_col=False):
    a, b = widen(a).ravel(), widen(b).ravel()
    lda = M if a_col else K
    ldb = K if b_col else N
    s = np.empty((M, N), dtype=np.float64)
    _load().oracle_gemm_absdot(_p(a), _p(b), _p(s), M, N, K, int(a_col), lda, int(b_col), ldb, N)
    return s


def conv2d(x, w, stride=(1, 1), pad=(0, 0), want_absdot=False):
    """x: [N,H,W,C], w: [K,R,S,C] float64 -> y [N,P,Q,K] float64 (cross-correlation,
    zero padding). With want_absdot also returns sum |x||w| per output."""
    x, w = widen(x), widen(w)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    sh, sw = stride
    ph, pw = pad
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    y = np.empty((N, P, Q, K), dtype=np.float64)
    ad = np.empty_like(y) if want_absdot else None
    _load().oracle_conv2d(_p(x), _p(w), _p(y), _p(ad) if want_absdot else None,
                          N, H, W, C, K, R, S, sh, sw, ph, pw)
    return (y, ad) if want_absdot else y


def round_f32(v) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.float32)
    _load().oracle_round_f32(_p(v), _p(out), v.size)
    return out


def round_bf16(v) -> np.ndarray:
    """float64 -> bf16 bit patterns (uint16), one round-to-nearest-even."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().oracle_round_bf16(_p(v), _p(out), v.size)
    return out
