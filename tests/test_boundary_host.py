"""Host-only checks of the C ABI: the library loads, exports every symbol declared in
include/perf.h, and rejects bad arguments before touching a device (so these run on a
machine without a GPU). No compute call is made here."""
import ctypes
import os
import re

import pytest

import paper_2511_03586_amd as perf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-null, 16-byte aligned fake device address; never dereferenced


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(perf.LIB_PATH):
        from paper_2511_03586_amd import build
        build.build(verbose=False)


def test_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "perf.h")).read()
    declared = set(re.findall(r"\b(perf_[a-z0-9_]+)\s*\(", header))
    declared -= {"perf_status", "perf_dtype", "perf_layout", "perf_stream"}
    assert {"perf_softmax", "perf_layernorm", "perf_gemm", "perf_conv2d", "perf_copy",
            "perf_status_string", "perf_version"} <= declared
    handle = ctypes.CDLL(perf.LIB_PATH)
    for name in declared:
        assert hasattr(handle, name), name
    assert declared == set(perf.SIGNATURES)


def test_version_and_status_strings():
    assert perf.version() >= 100
    names = {perf.status_string(s) for s in range(8)}
    assert len(names) == 8 and perf.status_string(0) == "ok"
    assert perf.status_string(99) == "unknown status"


def test_softmax_argument_errors():
    f = lambda **kw: perf.perf_softmax(**{**dict(x=FAKE, y=FAKE + 4096, rows=4, cols=8, ldx=8, ldy=8,
                                                 check=False), **kw})
    assert f(x=None) == perf.PERF_ERR_NULL and f(y=None) == perf.PERF_ERR_NULL
    assert f(rows=0) == perf.PERF_ERR_SHAPE and f(cols=-1) == perf.PERF_ERR_SHAPE
    assert f(ldx=7) == perf.PERF_ERR_SHAPE and f(ldy=3) == perf.PERF_ERR_SHAPE
    assert f(scale=float("inf")) == perf.PERF_ERR_SHAPE and f(scale=float("nan")) == perf.PERF_ERR_SHAPE
    assert f(x_dt=7) == perf.PERF_ERR_DTYPE and f(y_dt=-1) == perf.PERF_ERR_DTYPE
    assert f(x_dt=perf.PERF_BF16) == perf.PERF_ERR_UNSUPPORTED
    assert f(x=FAKE + 2) == perf.PERF_ERR_ALIGN
    with pytest.raises(perf.PerfError):
        perf.perf_softmax(None, FAKE, 1, 1, 1, 1)


def test_layernorm_argument_errors():
    base = dict(x=FAKE, gamma=FAKE + 4096, beta=FAKE + 8192, y=FAKE + 12288, mean_out=None, rstd_out=None,
                rows=4, cols=8, ldx=8, ldy=8, eps=1e-5, x_dt=perf.PERF_BF16, param_dt=perf.PERF_F32,
                y_dt=perf.PERF_BF16, check=False)
    f = lambda **kw: perf.perf_layernorm(**{**base, **kw})
    for k in ("x", "gamma", "beta", "y"):
        assert f(**{k: None}) == perf.PERF_ERR_NULL
    assert f(rows=0) == perf.PERF_ERR_SHAPE and f(cols=0) == perf.PERF_ERR_SHAPE
    assert f(ldx=4) == perf.PERF_ERR_SHAPE and f(eps=-1.0) == perf.PERF_ERR_SHAPE
    assert f(eps=float("nan")) == perf.PERF_ERR_SHAPE
    assert f(param_dt=2) == perf.PERF_ERR_DTYPE
    assert f(x=FAKE + 1) == perf.PERF_ERR_ALIGN and f(mean_out=FAKE + 2) == perf.PERF_ERR_ALIGN
    assert f(gamma=FAKE + 2) == perf.PERF_ERR_ALIGN      # fp32 params need 4-byte alignment


def test_gemm_argument_errors():
    base = dict(A=FAKE, B=FAKE + 4096, C=FAKE + 8192, M=4, N=4, K=8, la=perf.PERF_ROW_MAJOR, lda=8,
                lb=perf.PERF_COL_MAJOR, ldb=8, ldc=4, check=False)
    f = lambda **kw: perf.perf_gemm(**{**base, **kw})
    for k in ("A", "B", "C"):
        assert f(**{k: None}) == perf.PERF_ERR_NULL
    assert f(M=0) == perf.PERF_ERR_SHAPE and f(K=-3) == perf.PERF_ERR_SHAPE and f(batch=0) == perf.PERF_ERR_SHAPE
    assert f(lda=7) == perf.PERF_ERR_SHAPE and f(ldb=7) == perf.PERF_ERR_SHAPE and f(ldc=3) == perf.PERF_ERR_SHAPE
    assert f(la=perf.PERF_COL_MAJOR, lda=3) == perf.PERF_ERR_SHAPE    # col-major A needs lda >= M
    assert f(lb=perf.PERF_ROW_MAJOR, ldb=3) == perf.PERF_ERR_SHAPE    # row-major B needs ldb >= N
    assert f(batch=2, strideC=15) == perf.PERF_ERR_SHAPE              # C matrices would overlap
    assert f(strideA=-1) == perf.PERF_ERR_SHAPE and f(alpha=float("nan")) == perf.PERF_ERR_SHAPE
    assert f(la=2) == perf.PERF_ERR_LAYOUT and f(lb=-1) == perf.PERF_ERR_LAYOUT
    assert f(ab_dt=5) == perf.PERF_ERR_DTYPE
    assert f(ab_dt=perf.PERF_F32, c_dt=perf.PERF_BF16) == perf.PERF_ERR_UNSUPPORTED
    assert f(A=FAKE + 1) == perf.PERF_ERR_ALIGN and f(C=FAKE + 2) == perf.PERF_ERR_ALIGN


def test_conv2d_argument_errors():
    base = dict(x=FAKE, w=FAKE + 4096, y=FAKE + 8192, N=1, H=8, W=8, C=64, K=64, R=3, S=3, stride_h=1,
                stride_w=1, pad_h=1, pad_w=1, check=False)
    f = lambda **kw: perf.perf_conv2d(**{**base, **kw})
    for k in ("x", "w", "y"):
        assert f(**{k: None}) == perf.PERF_ERR_NULL
    for k in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w"):
        assert f(**{k: 0}) == perf.PERF_ERR_SHAPE
    assert f(pad_h=-1) == perf.PERF_ERR_SHAPE
    assert f(H=2, pad_h=0, R=3) == perf.PERF_ERR_SHAPE          # filter larger than padded image
    assert f(N=1 << 23, H=1 << 10, W=1 << 10, pad_h=0, pad_w=0, R=1, S=1) == perf.PERF_ERR_SHAPE  # too many pixels
    assert f(xw_dt=9) == perf.PERF_ERR_DTYPE
    assert f(x=FAKE + 1) == perf.PERF_ERR_ALIGN


def test_copy_argument_errors():
    assert perf.perf_copy(None, FAKE, 16, check=False) == perf.PERF_ERR_NULL
    assert perf.perf_copy(FAKE, FAKE + 64, -1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_copy(FAKE, FAKE + 64, 0, check=False) == perf.PERF_OK    # nothing to do, no launch


def test_mfma_probe_argument_errors():
    assert perf.perf_mfma_probe(None, 1, check=False) == perf.PERF_ERR_NULL
    assert perf.perf_mfma_probe(FAKE, 0, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_mfma_probe(FAKE, (1 << 24) + 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_mfma_probe(FAKE + 2, 1, check=False) == perf.PERF_ERR_ALIGN
    assert perf.perf_lds_probe(None, FAKE, 4, 16, 0, 1, check=False) == perf.PERF_ERR_NULL
    assert perf.perf_lds_probe(FAKE, FAKE, 5, 16, 0, 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_lds_probe(FAKE, FAKE, 4, 12, 0, 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_lds_probe(FAKE, FAKE, 4, 16, 0, 0, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_lds_probe(FAKE, FAKE, 4, 8, 1, 1, check=False) == perf.PERF_ERR_UNSUPPORTED
    assert perf.perf_lds_probe(FAKE, FAKE, 4, 16, 3, 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_lds_probe(FAKE + 4, FAKE, 4, 16, 0, 1, check=False) == perf.PERF_ERR_ALIGN
    # feed probe: src, src_bytes, cycles, sink, waves, mode, shared, span, iters
    assert perf.perf_feed_probe(None, 1 << 24, FAKE, FAKE, 4, 0, 0, 65536, 1, check=False) == perf.PERF_ERR_NULL
    assert perf.perf_feed_probe(FAKE, 1 << 24, FAKE, FAKE, 16, 0, 0, 65536, 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_feed_probe(FAKE, 1 << 24, FAKE, FAKE, 4, 4, 0, 65536, 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_feed_probe(FAKE, 1 << 24, FAKE, FAKE, 4, 0, 0, 65536 + 1024, 1, check=False) == perf.PERF_ERR_SHAPE   # not a power of two
    assert perf.perf_feed_probe(FAKE, (1 << 24) - 1, FAKE, FAKE, 4, 0, 0, 65536, 1, check=False) == perf.PERF_ERR_SHAPE   # 256 windows do not fit
    assert perf.perf_feed_probe(FAKE, 65536, FAKE, FAKE, 4, 0, 1, 65536, (1 << 14) + 1, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_feed_probe(FAKE + 8, 1 << 24, FAKE, FAKE, 4, 0, 0, 65536, 1, check=False) == perf.PERF_ERR_ALIGN
    assert perf.perf_mfma_probe_random(None, 1, check=False) == perf.PERF_ERR_NULL
    assert perf.perf_mfma_probe_random(FAKE, 0, check=False) == perf.PERF_ERR_SHAPE
    assert perf.perf_mfma_probe_random(FAKE + 2, 1, check=False) == perf.PERF_ERR_ALIGN


def test_gemm_softmax_argument_errors():
    def f(A=FAKE, B=FAKE + 4096, P=FAKE + 8192, M=8, N=8, K=32, lda=32, ldb=32, ldp=8, batch=1, sa=0, sb=0, sp=0,
          alpha=1.0, ab=perf.PERF_BF16, pd=perf.PERF_F32):
        return perf.perf_gemm_softmax(A, B, P, M, N, K, lda, ldb, ldp, batch, sa, sb, sp, alpha, ab, pd, check=False)
    assert f(A=None) == perf.PERF_ERR_NULL
    assert f(P=None) == perf.PERF_ERR_NULL
    assert f(M=0) == perf.PERF_ERR_SHAPE
    assert f(lda=31) == perf.PERF_ERR_SHAPE
    assert f(ldp=7) == perf.PERF_ERR_SHAPE
    assert f(batch=2, sp=63) == perf.PERF_ERR_SHAPE          # batches would overlap in P
    assert f(sa=-1) == perf.PERF_ERR_SHAPE
    assert f(alpha=float("inf")) == perf.PERF_ERR_SHAPE
    assert f(ab=7) == perf.PERF_ERR_DTYPE
    assert f(A=FAKE + 1) == perf.PERF_ERR_ALIGN
    assert f(K=33, lda=33, ldb=33, pd=perf.PERF_BF16) == perf.PERF_ERR_UNSUPPORTED   # two-operator path needs f32 P


def test_streaming_ops_argument_errors():
    r = lambda **k: perf.perf_rmsnorm(**{**dict(x=FAKE, gamma=FAKE + 4096, y=FAKE + 8192, rrms_out=None, rows=4, cols=8,
                                                 ldx=8, ldy=8, eps=1e-5, check=False), **k})
    assert r(x=None) == perf.PERF_ERR_NULL
    assert r(gamma=None) == perf.PERF_ERR_NULL
    assert r(cols=0) == perf.PERF_ERR_SHAPE
    assert r(ldy=7) == perf.PERF_ERR_SHAPE
    assert r(eps=-1.0) == perf.PERF_ERR_SHAPE
    assert r(x_dt=5) == perf.PERF_ERR_DTYPE
    assert r(x=FAKE + 1) == perf.PERF_ERR_ALIGN
    assert r(rrms_out=FAKE + 2) == perf.PERF_ERR_ALIGN
    m = lambda **k: perf.perf_reduce_mean(**{**dict(x=FAKE, y=FAKE + 4096, rows=4, cols=8, ldx=8, axis=1, check=False), **k})
    assert m(y=None) == perf.PERF_ERR_NULL
    assert m(rows=0) == perf.PERF_ERR_SHAPE
    assert m(ldx=7) == perf.PERF_ERR_SHAPE
    assert m(axis=2) == perf.PERF_ERR_SHAPE
    assert m(y_dt=3) == perf.PERF_ERR_DTYPE
    assert m(x=FAKE + 2) == perf.PERF_ERR_ALIGN
    mw = lambda **k: perf.perf_reduce_mean_ws(**{**dict(x=FAKE, y=FAKE + 4096, workspace=FAKE + 8192, rows=64, cols=8, ldx=8,
                                                        axis=0, check=False), **k})
    assert perf.perf_reduce_mean_workspace_bytes(64, 8, 0) == 2 * 8 * 4         # two row ranges of 32 rows
    assert perf.perf_reduce_mean_workspace_bytes(4096, 4096, 0) == 128 * 4096 * 4
    assert perf.perf_reduce_mean_workspace_bytes(4096, 4096, 0, perf.PERF_BF16) == 128 * 4096 * 4
    assert perf.perf_reduce_mean_workspace_bytes(64, 8, 1) == 0                 # axis 1 needs none
    assert perf.perf_reduce_mean_workspace_bytes(64, 7, 0) == 0                 # not whole 16-byte chunks: plain path
    assert perf.perf_reduce_mean_workspace_bytes(0, 8, 0) == -1
    assert perf.perf_reduce_mean_workspace_bytes(8, 8, 2) == -1
    assert perf.perf_reduce_mean_workspace_bytes(8, 8, 0, 7) == -1
    assert mw(x=None) == perf.PERF_ERR_NULL
    assert mw(workspace=None) == perf.PERF_ERR_NULL
    assert mw(workspace=FAKE + 8194) == perf.PERF_ERR_ALIGN
    assert mw(rows=0) == perf.PERF_ERR_SHAPE
    assert mw(ldx=7) == perf.PERF_ERR_SHAPE
    assert mw(axis=3) == perf.PERF_ERR_SHAPE
    assert mw(x_dt=9) == perf.PERF_ERR_DTYPE
    assert mw(x=FAKE + 2) == perf.PERF_ERR_ALIGN                                # falls to the plain path, which rejects it
    e = lambda **k: perf.perf_eltwise(**{**dict(op=perf.PERF_ADD, a=FAKE, b=FAKE + 4096, y=FAKE + 8192, n=16, check=False), **k})
    assert e(a=None) == perf.PERF_ERR_NULL
    assert e(b=None) == perf.PERF_ERR_NULL
    assert e(op=perf.PERF_RELU, b=None, n=0) == perf.PERF_OK        # relu needs no b; nothing to do, no launch
    assert e(op=7) == perf.PERF_ERR_UNSUPPORTED
    assert e(n=-1) == perf.PERF_ERR_SHAPE
    assert e(dt=4) == perf.PERF_ERR_DTYPE
    assert e(y=FAKE + 2) == perf.PERF_ERR_ALIGN
    assert e(n=0) == perf.PERF_OK


def test_variant_entry_points_refuse_without_touching_the_device():
    g = perf.perf_gemm_variant(FAKE, FAKE + 4096, FAKE + 8192, 64, 64, 64, perf.PERF_ROW_MAJOR, 64, perf.PERF_COL_MAJOR,
                               64, 64, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, 0, 32, check=False)
    assert g == perf.PERF_ERR_UNSUPPORTED                       # tile 0 is "library's choice": not a variant
    g = perf.perf_gemm_variant(FAKE, FAKE + 4096, FAKE + 8192, 64, 64, 64, perf.PERF_ROW_MAJOR, 64, perf.PERF_COL_MAJOR,
                               64, 64, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, 96, 32, check=False)
    assert g == perf.PERF_ERR_UNSUPPORTED
    g = perf.perf_gemm_variant(FAKE, FAKE + 4096, FAKE + 8192, 64, 64, 64, perf.PERF_ROW_MAJOR, 64, perf.PERF_ROW_MAJOR,
                               64, 64, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, 128, 32, check=False)
    assert g == perf.PERF_ERR_UNSUPPORTED                       # row-major B has no MFMA variant
    g = perf.perf_gemm_variant(None, FAKE, FAKE, 64, 64, 64, perf.PERF_ROW_MAJOR, 64, perf.PERF_COL_MAJOR,
                               64, 64, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, 128, 32, check=False)
    assert g == perf.PERF_ERR_NULL
    c = perf.perf_conv2d_variant(FAKE, FAKE + 4096, FAKE + 8192, 1, 8, 8, 3, 4, 3, 3, 1, 1, 1, 1, perf.PERF_BF16,
                                 perf.PERF_BF16, perf.CONV_WREG, check=False)
    assert c == perf.PERF_ERR_UNSUPPORTED
    c = perf.perf_conv2d_variant(FAKE, FAKE + 4096, FAKE + 8192, 1, 8, 8, 3, 4, 3, 3, 1, 1, 1, 1, perf.PERF_BF16,
                                 perf.PERF_BF16, 9, check=False)
    assert c == perf.PERF_ERR_UNSUPPORTED
    # the input-resident 3x3 kernel: stride 2; pixel ranges that would straddle images (33 x 35 outputs in
    # ranges of 32); rows too wide for the LDS; all refused before anything is launched
    for n, h, w_, st in [(2, 56, 56, 2), (3, 33, 35, 1), (1, 32, 1024, 1)]:
        c = perf.perf_conv2d_variant(FAKE, FAKE + 4096, FAKE + 8192, n, h, w_, 64, 128, 3, 3, st, st, 1, 1, perf.PERF_BF16,
                                     perf.PERF_BF16, perf.CONV_WRES, check=False)
        assert c == perf.PERF_ERR_UNSUPPORTED
    c = perf.perf_conv2d_variant(FAKE, FAKE + 4096, FAKE + 8192, 1, 8, 8, 3, 4, 3, 3, 0, 1, 1, 1, perf.PERF_BF16,
                                 perf.PERF_BF16, perf.CONV_DIRECT, check=False)
    assert c == perf.PERF_ERR_SHAPE


def test_batchnorm_argument_errors_and_workspace_size():
    f = lambda **k: perf.perf_batchnorm(**{**dict(x=FAKE, gamma=FAKE + 4096, beta=FAKE + 8192, y=FAKE + 12288,
                                                  mean_out=None, rstd_out=None, workspace=FAKE + 16384, N=2, C=3, H=4, W=5,
                                                  eps=1e-5, check=False), **k})
    for k in ("x", "gamma", "beta", "y", "workspace"):
        assert f(**{k: None}) == perf.PERF_ERR_NULL
    assert f(N=0) == perf.PERF_ERR_SHAPE and f(W=0) == perf.PERF_ERR_SHAPE
    assert f(N=4096, C=4096) == perf.PERF_ERR_SHAPE            # N*C planes ride on one grid dimension
    assert f(eps=float("nan")) == perf.PERF_ERR_SHAPE
    assert f(y_dt=6) == perf.PERF_ERR_DTYPE
    assert f(workspace=FAKE + 2) == perf.PERF_ERR_ALIGN
    assert f(x=FAKE + 1) == perf.PERF_ERR_ALIGN
    # 3 floats per segment of 16384 elements per plane, plus scale and mean per channel
    assert perf.perf_batchnorm_workspace_bytes(8, 64, 300, 300) == 4 * (3 * 64 * 8 * 6 + 2 * 64)
    assert perf.perf_batchnorm_workspace_bytes(1, 1, 1, 1) == 4 * (3 + 2)
    assert perf.perf_batchnorm_workspace_bytes(0, 1, 1, 1) == -1


def test_batchnorm_static_argument_errors_and_size_limit():
    f = lambda **k: perf.perf_batchnorm_static(**{**dict(x=FAKE, gamma=FAKE + 4096, beta=FAKE + 8192, y=FAKE + 12288,
                                                         mean_out=None, rstd_out=None, N=2, C=3, H=4, W=5, eps=1e-5,
                                                         check=False), **k})
    for k in ("x", "gamma", "beta", "y"):
        assert f(**{k: None}) == perf.PERF_ERR_NULL
    assert f(N=0) == perf.PERF_ERR_SHAPE and f(eps=-1.0) == perf.PERF_ERR_SHAPE
    assert f(x_dt=9) == perf.PERF_ERR_DTYPE
    assert f(y=FAKE + 2) == perf.PERF_ERR_ALIGN
    # 64 x 64 planes of 2048 x 2048 need 12 MiB of partials: beyond the 256 KiB built-in array,
    # refused before any device call
    assert perf.perf_batchnorm_static_max_bytes() == 256 * 1024
    assert perf.perf_batchnorm_workspace_bytes(64, 64, 2048, 2048) > perf.perf_batchnorm_static_max_bytes()
    assert f(N=64, C=64, H=2048, W=2048) == perf.PERF_ERR_UNSUPPORTED
    assert perf.perf_batchnorm_workspace_bytes(8, 3, 2048, 2048) <= perf.perf_batchnorm_static_max_bytes()


def test_stream_probe_argument_errors():
    f = lambda **k: perf.perf_stream_probe(**{**dict(src=FAKE, dst=FAKE + 65536, nbytes=4096, mode=0, unroll=4, threads=256,
                                                     grid=0, policy=3, check=False), **k})
    assert f(src=None) == perf.PERF_ERR_NULL and f(dst=None) == perf.PERF_ERR_NULL
    for bad in (dict(nbytes=0), dict(nbytes=24), dict(mode=3), dict(threads=96), dict(grid=-1), dict(policy=4)):
        assert f(**bad) == perf.PERF_ERR_SHAPE, bad
    assert f(src=FAKE + 8) == perf.PERF_ERR_ALIGN
    assert f(unroll=3) == perf.PERF_ERR_UNSUPPORTED
