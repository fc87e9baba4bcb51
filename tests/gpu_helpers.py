"""Glue for the GPU parity tests: numpy <-> device buffers (torch is only used for device
memory and the stream) and calls through the C ABI binding. No operator arithmetic here."""
import numpy as np
import torch

import paper_2511_03586_amd as perf


def dev(a: np.ndarray) -> torch.Tensor:
    """Copy a numpy array to the GPU bit-for-bit (uint16 bf16 patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def host(t: torch.Tensor, bf16: bool = False) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint16) if bf16 else a


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def dt(bf16: bool) -> int:
    return perf.PERF_BF16 if bf16 else perf.PERF_F32


def run_softmax(x: np.ndarray, scale: float = 1.0, ldx=None, ldy=None, inplace=False, offset=0) -> np.ndarray:
    rows, cols = x.shape
    ldx = ldx or cols
    ldy = ldx if inplace else (ldy or cols)
    xb = np.zeros(rows * ldx + offset, dtype=np.float32)
    xb[offset:].reshape(rows, ldx)[:, :cols] = x
    xd = dev(xb)
    yd = xd if inplace else torch.full((rows * ldy + offset,), 7.0, dtype=torch.float32, device="cuda")
    perf.perf_softmax(xd.data_ptr() + 4 * offset, yd.data_ptr() + 4 * offset, rows, cols, ldx, ldy,
                      perf.PERF_F32, perf.PERF_F32, scale, stream())
    torch.cuda.synchronize()
    out = host(yd)
    if not inplace:
        pad = out[offset:].reshape(rows, ldy)[:, cols:]
        assert np.all(pad == 7.0), "kernel wrote into the row padding"
        assert np.all(out[:offset] == 7.0)
    return out[offset:].reshape(rows, ldy)[:, :cols].copy()


def run_layernorm(x, gamma, beta, eps, x_bf16, p_bf16, y_bf16, want_stats=True, ldx=None, ldy=None,
                  inplace=False, offset=0):
    """x: float32 array, or uint16 bf16 bits when x_bf16. Returns (y, mean, rstd); y is
    uint16 bits when y_bf16."""
    rows, cols = x.shape
    ldx = ldx or cols
    ldy = ldx if inplace else (ldy or cols)
    xb = np.zeros(rows * ldx + offset, dtype=x.dtype)
    xb[offset:].reshape(rows, ldx)[:, :cols] = x
    xd = dev(xb)
    ydtype = torch.int16 if y_bf16 else torch.float32
    yd = xd if inplace else torch.zeros(rows * ldy + offset, dtype=ydtype, device="cuda")
    gd, bd = dev(gamma), dev(beta)
    md = torch.zeros(rows, dtype=torch.float32, device="cuda") if want_stats else None
    rd = torch.zeros(rows, dtype=torch.float32, device="cuda") if want_stats else None
    xs, ys = (2 if x_bf16 else 4), (2 if y_bf16 else 4)
    perf.perf_layernorm(xd.data_ptr() + xs * offset, gd.data_ptr(), bd.data_ptr(), yd.data_ptr() + ys * offset,
                        md.data_ptr() if want_stats else None, rd.data_ptr() if want_stats else None,
                        rows, cols, ldx, ldy, eps, dt(x_bf16), dt(p_bf16), dt(y_bf16), stream())
    torch.cuda.synchronize()
    out = host(yd, y_bf16)
    if not inplace:
        assert np.all(out[offset:].reshape(rows, ldy)[:, cols:] == 0), "kernel wrote into the row padding"
    y = out[offset:].reshape(rows, ldy)[:, :cols].copy()
    return y, (host(md) if want_stats else None), (host(rd) if want_stats else None)


def run_gemm(a, b, M, N, K, a_col=False, b_col=True, alpha=1.0, batch=1, ab_bf16=True, c_bf16=False,
             lda=None, ldb=None, ldc=None, tile=0, kstep=0):
    """a, b: storage arrays (uint16 bits or float32), densely packed per batch with the
    given leading dimensions. Returns C as [batch, M, N] (uint16 bits if c_bf16)."""
    lda = lda or (M if a_col else K)
    ldb = ldb or (K if b_col else N)
    ldc = ldc or N
    sa = lda * (K if a_col else M)
    sb = ldb * (N if b_col else K)
    sc = M * ldc
    ad, bd = dev(np.ascontiguousarray(a).ravel()), dev(np.ascontiguousarray(b).ravel())
    assert ad.numel() >= batch * sa and bd.numel() >= batch * sb
    cd = torch.zeros(batch * sc, dtype=torch.int16 if c_bf16 else torch.float32, device="cuda")
    la = perf.PERF_COL_MAJOR if a_col else perf.PERF_ROW_MAJOR
    lb = perf.PERF_COL_MAJOR if b_col else perf.PERF_ROW_MAJOR
    if tile or kstep:  # a named kernel variant instead of the library's own choice
        perf.perf_gemm_variant(ad.data_ptr(), bd.data_ptr(), cd.data_ptr(), M, N, K, la, lda, lb, ldb, ldc,
                               batch, sa, sb, sc, alpha, dt(ab_bf16), dt(c_bf16), tile, kstep, stream())
    else:
        perf.perf_gemm(ad.data_ptr(), bd.data_ptr(), cd.data_ptr(), M, N, K, la, lda, lb, ldb, ldc,
                       batch, sa, sb, sc, alpha, dt(ab_bf16), dt(c_bf16), stream())
    torch.cuda.synchronize()
    c = host(cd, c_bf16).reshape(batch, M, ldc)
    assert np.all(c[:, :, N:] == 0), "kernel wrote into the row padding of C"
    return c[:, :, :N].copy()


def run_gemm_softmax(a, b, M, N, K, alpha=1.0, batch=1, ab_bf16=True, p_bf16=False, lda=None, ldb=None, ldp=None):
    """a: [batch] x M rows of lda, b: [batch] x N rows of ldb (storage arrays). Returns P [batch, M, N]."""
    lda, ldb, ldp = lda or K, ldb or K, ldp or N
    sa, sb, sp = M * lda, N * ldb, M * ldp
    ad, bd = dev(np.ascontiguousarray(a).ravel()), dev(np.ascontiguousarray(b).ravel())
    assert ad.numel() >= batch * sa and bd.numel() >= batch * sb
    pd = torch.zeros(batch * sp, dtype=torch.int16 if p_bf16 else torch.float32, device="cuda")
    perf.perf_gemm_softmax(ad.data_ptr(), bd.data_ptr(), pd.data_ptr(), M, N, K, lda, ldb, ldp, batch, sa, sb, sp,
                           alpha, dt(ab_bf16), dt(p_bf16), stream())
    torch.cuda.synchronize()
    p = host(pd, p_bf16).reshape(batch, M, ldp)
    assert np.all(p[:, :, N:] == 0), "kernel wrote into the row padding of P"
    return p[:, :, :N].copy()


def run_conv2d(x, w, stride=(1, 1), pad=(0, 0), xw_bf16=True, y_bf16=True, variant=0):
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    xd, wd = dev(x), dev(w)
    yd = torch.zeros(N * P * Q * K, dtype=torch.int16 if y_bf16 else torch.float32, device="cuda")
    if variant:
        perf.perf_conv2d_variant(xd.data_ptr(), wd.data_ptr(), yd.data_ptr(), N, H, W, C, K, R, S, stride[0], stride[1],
                                 pad[0], pad[1], dt(xw_bf16), dt(y_bf16), variant, stream())
    else:
        perf.perf_conv2d(xd.data_ptr(), wd.data_ptr(), yd.data_ptr(), N, H, W, C, K, R, S, stride[0], stride[1],
                         pad[0], pad[1], dt(xw_bf16), dt(y_bf16), stream())
    torch.cuda.synchronize()
    return host(yd, y_bf16).reshape(N, P, Q, K)
