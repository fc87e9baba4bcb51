"""The diagnostic builds with cycle-counter stamps (csrc/timeline.h): the stamped kernels must compute what
the product kernels compute, bit for bit, and their stamps must be ordered like the phases they mark."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _libs():
    from paper_2511_03586_amd import build as B, timeline as T
    paths = [B.timeline_lib(1), B.timeline_lib(2)]
    if not all(os.path.exists(p) for p in paths):
        pytest.skip("diagnostic libraries not built (python -m paper_2511_03586_amd.build --timeline)")
    return T, [T._load(p) for p in paths]


@pytest.mark.parametrize("variant", [8, 6])
def test_stamped_convolution_matches_the_product_kernel_and_orders_its_phases(variant):
    import torch
    import paper_2511_03586_amd as perf
    T, libs = _libs()
    N, H, W, C, K = 32, 56, 56, 64, 128
    torch.manual_seed(3)
    x = torch.randint(-4, 5, (N, H, W, C), device="cuda").to(torch.bfloat16)
    w = torch.randint(-3, 4, (K, 3, 3, C), device="cuda").to(torch.bfloat16)
    st = torch.cuda.current_stream().cuda_stream
    want = torch.empty(N, H, W, K, device="cuda", dtype=torch.bfloat16)
    perf.perf_conv2d_variant(x.data_ptr(), w.data_ptr(), want.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 1, 1,
                             perf.PERF_BF16, perf.PERF_BF16, variant, st)
    for level, lib in enumerate(libs, start=1):
        got = torch.zeros_like(want)
        rc = lib.perf_conv2d_variant(x.data_ptr(), w.data_ptr(), got.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 1, 1, 1, 1, variant, st)
        assert rc == 0
        buf = T._fetch(lib.perf_timeline_fetch_conv)
        assert torch.equal(got, want)
        for role in (0, 1):
            end, ticks = buf[:, role, 0], buf[:, role, 1]
            assert np.all(end > 0) and np.all(ticks > 0)          # every workgroup reported
            phases = [buf[:, role, s] for s in (2, 3, 4)]
            assert np.all(phases[0] > 0) and np.all(phases[0] <= phases[1]) and np.all(phases[1] <= phases[2])
            assert np.all(phases[2] < end)
            ghz = end / (ticks * 10.0)
            assert np.all(ghz > 0.5) and np.all(ghz < 3.0)
        steps = buf[:, 0, 8 + 2:8 + 13]
        if level == 2:
            assert np.all(np.diff(steps, axis=1) > 0)             # one stamp per step, in order
        else:
            assert not steps.any()
        assert not T._fetch(lib.perf_timeline_fetch_conv).any()  # fetching clears the buffer


def test_stamped_gemm_orders_its_phases():
    import torch
    T, libs = _libs()
    buf, us = T.gemm_timeline(torch, libs[0], zeros=False, launches=4)
    t2, t3, t4, end = (buf[:, 0, s] for s in (2, 3, 4, 0))
    assert np.all(t2 > 0) and np.all(t2 < t3) and np.all(t3 < t4) and np.all(t4 <= end)
    assert np.all(t3 - t2 >= 131072)  # the main loop cannot take fewer cycles than its MFMAs
    assert 50.0 < us < 500.0
