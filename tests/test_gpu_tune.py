"""GPU: the variant entry points agree with the default path, and the timing-driven search
visits, validates and ranks them."""
import numpy as np
import pytest

import oracle
import paper_2511_03586_amd as perf
from paper_2511_03586_amd import tune
from workloads import configs
from tests import gpu_helpers as G
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_gemm_variants_match_the_oracle():
    import torch
    wl = configs.GemmWorkload(M=300, N=260, K=192)
    d = wl.make()
    ad, bd = G.dev(d["a_bf16"]), G.dev(d["b_bf16"])
    a64, b64 = oracle.widen(d["a_bf16"], True), oracle.widen(d["b_bf16"], True)
    ref = oracle.gemm(a64, b64, wl.M, wl.N, wl.K, b_col=True)
    s = oracle.gemm_absdot(a64, b64, wl.M, wl.N, wl.K, b_col=True)
    for tile, kstep in tune.GEMM_SPACE:
        c = torch.zeros(wl.M * wl.N, dtype=torch.float32, device="cuda")
        perf.perf_gemm_variant(ad.data_ptr(), bd.data_ptr(), c.data_ptr(), wl.M, wl.N, wl.K, perf.PERF_ROW_MAJOR, wl.K,
                               perf.PERF_COL_MAJOR, wl.K, wl.N, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, tile,
                               kstep, G.stream())
        torch.cuda.synchronize()
        P.assert_contraction_close(c.cpu().numpy().reshape(wl.M, wl.N), ref, s, wl.K)
    # K = 96 is not a multiple of 64: that variant must refuse, not compute
    rc = perf.perf_gemm_variant(ad.data_ptr(), bd.data_ptr(), c.data_ptr(), wl.M, wl.N, 96, perf.PERF_ROW_MAJOR, wl.K,
                                perf.PERF_COL_MAJOR, wl.K, wl.N, 1, 0, 0, 0, 1.0, perf.PERF_BF16, perf.PERF_F32, 128, 64,
                                G.stream(), check=False)
    assert rc == perf.PERF_ERR_UNSUPPORTED


def test_search_gemm_visits_validates_and_ranks():
    out = tune.search_gemm(768, 1024, 1024, iters=10, warmup=2)
    assert len(out["results"]) == len(tune.GEMM_SPACE)
    assert all(r["status"] == "ok" and r["max_rel_diff"] <= 1e-5 for r in out["results"])
    assert out["best"]["us"] == min(r["us"] for r in out["results"])
    assert out["best"]["us"] <= out["default_us"] * 1.5       # the library's rule is not far from the best variant (timing noise allowed for)
    sub = tune.search_gemm(256, 256, 128, iters=5, warmup=1, sample=2, seed=3)
    assert len(sub["results"]) == 2


def test_search_conv_families():
    out = tune.search_conv(4, 56, 56, 64, 128, 3, 3, iters=10, warmup=2)
    by = {r["variant"]: r for r in out["results"]}
    assert by[perf.CONV_WREG]["status"] == "ok" and by[perf.CONV_MFMA]["status"] == "ok"
    assert by[perf.CONV_DIRECT]["status"] == "ok"
    assert out["best"]["variant"] in (perf.CONV_WREG, perf.CONV_MFMA)
    out = tune.search_conv(2, 128, 128, 3, 10, 5, 5, pad=2, iters=5, warmup=1)
    by = {r["variant"]: r for r in out["results"]}
    assert by[perf.CONV_WREG]["status"] == "unsupported" and by[perf.CONV_MFMA]["status"] == "unsupported"
    assert by[perf.CONV_SMALLC]["status"] == "ok" and by[perf.CONV_DIRECT]["status"] == "ok"
    assert by[perf.CONV_ROWMFMA]["status"] == "ok"
    assert out["best"]["variant"] in (perf.CONV_ROWMFMA, perf.CONV_SMALLC)
