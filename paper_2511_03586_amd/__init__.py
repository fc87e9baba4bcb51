"""MI355X (gfx950) operator library: thin ctypes binding over ``libperf.so``.

The functions here have the names and arguments of the C ABI in ``include/perf.h`` and do
argument marshalling only; every step of every operator runs in the HIP kernels. torch is
used by callers for device memory and streams. The library is loaded lazily and loading
fails loudly: there is no fallback path of any kind.
"""
from __future__ import annotations

import ctypes
import os

PERF_OK = 0
PERF_ERR_NULL, PERF_ERR_SHAPE, PERF_ERR_DTYPE, PERF_ERR_LAYOUT = 1, 2, 3, 4
PERF_ERR_ALIGN, PERF_ERR_UNSUPPORTED, PERF_ERR_LAUNCH = 5, 6, 7
PERF_F32, PERF_BF16 = 0, 1
PERF_ROW_MAJOR, PERF_COL_MAJOR = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libperf.so")
_lib = None

_i64, _f32, _ptr, _int = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int

SIGNATURES = {
    "perf_softmax": (_int, [_ptr, _ptr, _i64, _i64, _i64, _i64, _int, _int, _f32, _ptr]),
    "perf_layernorm": (_int, [_ptr, _ptr, _ptr, _ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _f32,
                              _int, _int, _int, _ptr]),
    "perf_gemm": (_int, [_ptr, _ptr, _ptr, _i64, _i64, _i64, _int, _i64, _int, _i64, _i64,
                         _i64, _i64, _i64, _i64, _f32, _int, _int, _ptr]),
    "perf_conv2d": (_int, [_ptr, _ptr, _ptr] + [_i64] * 11 + [_int, _int, _ptr]),
    "perf_gemm_softmax": (_int, [_ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _f32,
                                 _int, _int, _ptr]),
    "perf_rmsnorm": (_int, [_ptr, _ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _f32, _int, _int, _int, _ptr]),
    "perf_reduce_mean": (_int, [_ptr, _ptr, _i64, _i64, _i64, _int, _int, _int, _ptr]),
    "perf_reduce_mean_workspace_bytes": (_i64, [_i64, _i64, _int, _int]),
    "perf_reduce_mean_ws": (_int, [_ptr, _ptr, _ptr, _i64, _i64, _i64, _int, _int, _int, _ptr]),
    "perf_eltwise": (_int, [_int, _ptr, _ptr, _ptr, _i64, _int, _ptr]),
    "perf_softmax_variant": (_int, [_ptr, _ptr, _i64, _i64, _i64, _i64, _int, _int, _f32, _int, _int, _i64, _ptr]),
    "perf_layernorm_variant": (_int, [_ptr, _ptr, _ptr, _ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _f32,
                                      _int, _int, _int, _int, _i64, _ptr]),
    "perf_gemm_variant": (_int, [_ptr, _ptr, _ptr, _i64, _i64, _i64, _int, _i64, _int, _i64, _i64, _i64, _i64, _i64, _i64,
                                 _f32, _int, _int, _int, _int, _ptr]),
    "perf_conv2d_variant": (_int, [_ptr, _ptr, _ptr] + [_i64] * 11 + [_int, _int, _int, _ptr]),
    "perf_batchnorm_workspace_bytes": (_i64, [_i64, _i64, _i64, _i64]),
    "perf_batchnorm": (_int, [_ptr, _ptr, _ptr, _ptr, _ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _f32, _int, _int, _int,
                              _ptr]),
    "perf_batchnorm_static_max_bytes": (_i64, []),
    "perf_batchnorm_static": (_int, [_ptr, _ptr, _ptr, _ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _f32, _int, _int, _int,
                                     _ptr]),
    "perf_copy": (_int, [_ptr, _ptr, _i64, _ptr]),
    "perf_stream_probe": (_int, [_ptr, _ptr, _i64, _int, _int, _int, _i64, _int, _ptr]),
    "perf_mfma_probe": (_int, [_ptr, _i64, _ptr]),
    "perf_mfma_probe_random": (_int, [_ptr, _i64, _ptr]),
    "perf_lds_probe": (_int, [_ptr, _ptr, _int, _int, _int, _i64, _ptr]),
    "perf_feed_probe": (_int, [_ptr, _i64, _ptr, _ptr, _int, _int, _int, _i64, _i64, _ptr]),
    "perf_status_string": (ctypes.c_char_p, [_int]),
    "perf_version": (_int, []),
}


class PerfError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """The loaded library. Raises if ``libperf.so`` has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with "
                               f"`python -m paper_2511_03586_amd.build` (there is no fallback path)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def status_string(status: int) -> str:
    return lib().perf_status_string(int(status)).decode()


def version() -> int:
    return lib().perf_version()


def _check(fn: str, status: int, check: bool) -> int:
    if check and status != PERF_OK:
        raise PerfError(fn, status)
    return status


def perf_softmax(x, y, rows, cols, ldx, ldy, x_dt=PERF_F32, y_dt=PERF_F32, scale=1.0, stream=None,
                 check=True) -> int:
    """x, y: device addresses (ints). See ``perf_softmax`` in include/perf.h."""
    return _check("perf_softmax", lib().perf_softmax(x, y, rows, cols, ldx, ldy, x_dt, y_dt, scale, stream), check)


def perf_layernorm(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps, x_dt, param_dt, y_dt,
                   stream=None, check=True) -> int:
    return _check("perf_layernorm",
                  lib().perf_layernorm(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps,
                                       x_dt, param_dt, y_dt, stream), check)


def perf_gemm(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch=1, strideA=0, strideB=0, strideC=0, alpha=1.0,
              ab_dt=PERF_BF16, c_dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_gemm",
                  lib().perf_gemm(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch, strideA, strideB, strideC,
                                  alpha, ab_dt, c_dt, stream), check)


def perf_gemm_softmax(A, B, P, M, N, K, lda, ldb, ldp, batch=1, strideA=0, strideB=0, strideP=0, alpha=1.0,
                      ab_dt=PERF_BF16, p_dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_gemm_softmax",
                  lib().perf_gemm_softmax(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP,
                                          alpha, ab_dt, p_dt, stream), check)


def perf_conv2d(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, xw_dt=PERF_BF16,
                y_dt=PERF_BF16, stream=None, check=True) -> int:
    return _check("perf_conv2d",
                  lib().perf_conv2d(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w,
                                    xw_dt, y_dt, stream), check)


def perf_gemm_variant(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch, strideA, strideB, strideC, alpha, ab_dt, c_dt,
                      tile, kstep, stream=None, check=True) -> int:
    return _check("perf_gemm_variant",
                  lib().perf_gemm_variant(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch, strideA, strideB, strideC,
                                          alpha, ab_dt, c_dt, tile, kstep, stream), check)


def perf_softmax_variant(x, y, rows, cols, ldx, ldy, x_dt, y_dt, scale, rows_per_wave, waves_per_row, grid,
                         stream=None, check=True) -> int:
    return _check("perf_softmax_variant",
                  lib().perf_softmax_variant(x, y, rows, cols, ldx, ldy, x_dt, y_dt, scale, rows_per_wave, waves_per_row,
                                             grid, stream), check)


def perf_layernorm_variant(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps, x_dt, param_dt, y_dt,
                           waves_per_row, grid, stream=None, check=True) -> int:
    return _check("perf_layernorm_variant",
                  lib().perf_layernorm_variant(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps,
                                               x_dt, param_dt, y_dt, waves_per_row, grid, stream), check)


CONV_WREG, CONV_MFMA, CONV_SMALLC, CONV_DIRECT, CONV_ROWMFMA, CONV_WRES, CONV_F32MFMA, CONV_WSPLIT = 1, 2, 3, 4, 5, 6, 7, 8


def perf_conv2d_variant(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, xw_dt, y_dt, variant,
                        stream=None, check=True) -> int:
    return _check("perf_conv2d_variant",
                  lib().perf_conv2d_variant(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, xw_dt, y_dt,
                                            variant, stream), check)


PERF_ADD, PERF_MUL, PERF_RELU = 0, 1, 2


def perf_rmsnorm(x, gamma, y, rrms_out, rows, cols, ldx, ldy, eps, x_dt=PERF_BF16, param_dt=PERF_F32,
                 y_dt=PERF_BF16, stream=None, check=True) -> int:
    return _check("perf_rmsnorm",
                  lib().perf_rmsnorm(x, gamma, y, rrms_out, rows, cols, ldx, ldy, eps, x_dt, param_dt, y_dt, stream),
                  check)


def perf_reduce_mean(x, y, rows, cols, ldx, axis, x_dt=PERF_F32, y_dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_reduce_mean", lib().perf_reduce_mean(x, y, rows, cols, ldx, axis, x_dt, y_dt, stream), check)


def perf_reduce_mean_workspace_bytes(rows, cols, axis, x_dt=PERF_F32) -> int:
    return int(lib().perf_reduce_mean_workspace_bytes(rows, cols, axis, x_dt))


def perf_reduce_mean_ws(x, y, workspace, rows, cols, ldx, axis, x_dt=PERF_F32, y_dt=PERF_F32, stream=None,
                        check=True) -> int:
    return _check("perf_reduce_mean_ws",
                  lib().perf_reduce_mean_ws(x, y, workspace, rows, cols, ldx, axis, x_dt, y_dt, stream), check)


def perf_eltwise(op, a, b, y, n, dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_eltwise", lib().perf_eltwise(op, a, b, y, n, dt, stream), check)


def perf_batchnorm_workspace_bytes(N, C, H, W) -> int:
    return int(lib().perf_batchnorm_workspace_bytes(N, C, H, W))


def perf_batchnorm(x, gamma, beta, y, mean_out, rstd_out, workspace, N, C, H, W, eps, x_dt=PERF_F32,
                   param_dt=PERF_F32, y_dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_batchnorm",
                  lib().perf_batchnorm(x, gamma, beta, y, mean_out, rstd_out, workspace, N, C, H, W, eps, x_dt,
                                       param_dt, y_dt, stream), check)


def perf_batchnorm_static_max_bytes() -> int:
    return int(lib().perf_batchnorm_static_max_bytes())


def perf_batchnorm_static(x, gamma, beta, y, mean_out, rstd_out, N, C, H, W, eps, x_dt=PERF_F32,
                          param_dt=PERF_F32, y_dt=PERF_F32, stream=None, check=True) -> int:
    return _check("perf_batchnorm_static",
                  lib().perf_batchnorm_static(x, gamma, beta, y, mean_out, rstd_out, N, C, H, W, eps, x_dt,
                                              param_dt, y_dt, stream), check)


def perf_copy(src, dst, nbytes, stream=None, check=True) -> int:
    return _check("perf_copy", lib().perf_copy(src, dst, nbytes, stream), check)


def perf_stream_probe(src, dst, nbytes, mode, unroll, threads, grid, policy, stream=None, check=True) -> int:
    return _check("perf_stream_probe",
                  lib().perf_stream_probe(src, dst, nbytes, mode, unroll, threads, grid, policy, stream), check)


MFMA_PROBE_SINK_FLOATS = 4096
MFMA_PROBE_FLOP_PER_ITER = 4096 * 32 * 32768


def perf_mfma_probe(sink, iters, stream=None, check=True) -> int:
    return _check("perf_mfma_probe", lib().perf_mfma_probe(sink, iters, stream), check)


def perf_mfma_probe_random(sink, iters, stream=None, check=True) -> int:
    return _check("perf_mfma_probe_random", lib().perf_mfma_probe_random(sink, iters, stream), check)


def perf_lds_probe(cycles, sink, waves, bytes_per_lane, with_mfma, iters, stream=None, check=True) -> int:
    return _check("perf_lds_probe", lib().perf_lds_probe(cycles, sink, waves, bytes_per_lane, with_mfma, iters, stream), check)


def perf_feed_probe(src, src_bytes, cycles, sink, waves, mode, shared, span, iters, stream=None, check=True) -> int:
    return _check("perf_feed_probe",
                  lib().perf_feed_probe(src, src_bytes, cycles, sink, waves, mode, shared, span, iters, stream), check)
