"""GPU: perf_batchnorm_static (the entry point that allocates nothing; its scratch is a fixed
device array inside the library) against perf_batchnorm with a caller workspace. Both run the
same kernels, so the bar is bit equality of y, mean and rstd; the first result is also checked
against the CPU oracle at the batchnorm tolerances (1e-5). Two calls in a row, the second on a
smaller input, so that stale scratch from the first call would show."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_03586_amd as perf
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu


def _inputs(N, C, H, W, seed):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((N, C, H, W)) * g.uniform(0.5, 3.0, C)[None, :, None, None]
         + g.uniform(-3, 3, C)[None, :, None, None]).astype(np.float32)
    return x, g.uniform(0.5, 1.5, C).astype(np.float32), (g.standard_normal(C) * 0.3).astype(np.float32)


def _call(static, x, gamma, beta, eps=1e-5):
    N, C, H, W = x.shape
    xd, gd, bd = G.dev(x.ravel()), G.dev(gamma), G.dev(beta)
    yd = torch.zeros(x.size, dtype=torch.float32, device="cuda")
    md = torch.zeros(C, dtype=torch.float32, device="cuda")
    rd = torch.zeros(C, dtype=torch.float32, device="cuda")
    if static:
        perf.perf_batchnorm_static(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), yd.data_ptr(), md.data_ptr(),
                                   rd.data_ptr(), N, C, H, W, eps, perf.PERF_F32, perf.PERF_F32, perf.PERF_F32, G.stream())
    else:
        ws = torch.zeros(perf.perf_batchnorm_workspace_bytes(N, C, H, W) // 4, dtype=torch.float32, device="cuda")
        perf.perf_batchnorm(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), yd.data_ptr(), md.data_ptr(), rd.data_ptr(),
                            ws.data_ptr(), N, C, H, W, eps, perf.PERF_F32, perf.PERF_F32, perf.PERF_F32, G.stream())
    torch.cuda.synchronize()
    return yd.cpu().numpy().reshape(x.shape), md.cpu().numpy(), rd.cpu().numpy()


def test_static_scratch_entry_point_two_calls_second_smaller():
    for shape, seed in (((8, 16, 150, 150), 11), ((2, 5, 33, 47), 12)):    # 2 segments per plane, then 1 ragged
        x, gamma, beta = _inputs(*shape, seed)
        assert perf.perf_batchnorm_workspace_bytes(*shape) <= perf.perf_batchnorm_static_max_bytes()
        ys, ms, rs = _call(True, x, gamma, beta)
        yw, mw, rw = _call(False, x, gamma, beta)
        assert np.array_equal(ys, yw) and np.array_equal(ms, mw) and np.array_equal(rs, rw), shape
        ref, mref, rref = oracle.batchnorm(x, gamma, beta, float(np.float32(1e-5)))
        rms = np.sqrt(np.mean(ref ** 2, axis=(0, 2, 3), keepdims=True))
        assert np.max(np.abs(ys - ref) / np.maximum(np.abs(ref), rms)) <= 1e-5
        assert np.max(np.abs(ms - mref) / np.maximum(np.abs(mref), 1e-3)) <= 1e-5
        assert np.max(np.abs(rs - rref) / rref) <= 1e-5
