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
    for tile, kstep in [(t, k) for t in (64, 128, 256) for k in (32, 64)] + [(64, 33), (128, 33), (256, 65)]:
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


def _oracle_gemm_validator(inputs, M, N, K):
    """Candidate outputs are checked against the CPU oracle on the search's own seeded operands."""
    a64, b64 = oracle.widen(inputs["a_bf16"], True), oracle.widen(inputs["b_bf16"], True)
    ref = oracle.gemm(a64, b64, M, N, K, b_col=True)
    s = oracle.gemm_absdot(a64, b64, M, N, K, b_col=True)

    def validate(out):
        try:
            gate = P.assert_contraction_close(out.reshape(M, N), ref, s, K)
        except AssertionError:
            return False, float("inf")
        return True, float(gate)
    return validate


def test_search_gemm_visits_validates_and_ranks():
    M, N, K = 768, 1024, 1024
    probe = tune.search_gemm(M, N, K, iters=2, warmup=1, strategy="random", budget=1)     # (its seeded operands)
    out = tune.search_gemm(M, N, K, iters=10, warmup=2, validate=_oracle_gemm_validator(probe["inputs"], M, N, K))
    assert out["visited"] == len(tune.GEMM_AXES["tile"]) * len(tune.GEMM_AXES["kstep"])
    ran = [r for r in out["results"] if r["status"] == "ok"]
    assert len(ran) == 9 and not any(r["status"] == "rejected" for r in out["results"])   # 3 tiles x {32, 64}, 2 deep rings, 1 on 32x32x16
    assert out["best"]["us"] == min(r["us"] for r in ran)
    # the library's shape rule is not far from the best variant (timing noise allowed for)
    assert out["default_us"] <= out["best"]["us"] * 1.5
    sub = tune.search_gemm(256, 256, 128, iters=5, warmup=1, strategy="random", budget=2, seed=3)
    assert sub["visited"] == 2


def test_a_wrong_candidate_is_rejected():
    # a validator that demands the impossible rejects every candidate: nothing is timed or ranked
    out = tune.search_gemm(256, 256, 128, iters=2, warmup=1, validate=lambda o: (False, 1.0))
    assert out["best"] is None and all(r["status"] in ("rejected", "unsupported") for r in out["results"])


def test_search_conv_families():
    out = tune.search_conv(4, 56, 56, 64, 128, 3, 3, iters=10, warmup=2)
    by = {r["variant"]["variant"]: r for r in out["results"]}
    assert by[perf.CONV_WREG]["status"] == "ok" and by[perf.CONV_MFMA]["status"] == "ok"
    assert by[perf.CONV_DIRECT]["status"] == "ok" and by[perf.CONV_WSPLIT]["status"] == "ok"
    assert out["best"]["variant"]["variant"] in (perf.CONV_WSPLIT, perf.CONV_WRES, perf.CONV_WREG, perf.CONV_MFMA)
    out = tune.search_conv(2, 128, 128, 3, 10, 5, 5, pad=2, iters=5, warmup=1)
    by = {r["variant"]["variant"]: r for r in out["results"]}
    assert by[perf.CONV_WREG]["status"] == "unsupported" and by[perf.CONV_MFMA]["status"] == "unsupported"
    assert by[perf.CONV_SMALLC]["status"] == "ok" and by[perf.CONV_DIRECT]["status"] == "ok"
    assert by[perf.CONV_ROWMFMA]["status"] == "ok"


def test_softmax_and_layernorm_variants_match_the_oracle():
    import torch
    rows, cols = 300, 1024
    x = configs.SoftmaxWorkload(rows=rows, cols=cols).make()["x"]
    ref = oracle.softmax(x)
    xd = G.dev(x)
    ran = 0
    for wpr, rpw, grid in [(1, 1, 0), (1, 2, 0), (1, 4, 0), (1, 2, 7), (4, 0, 0), (4, 0, 5), (16, 0, 0), (16, 0, 3), (0, 0, 9)]:
        yd = torch.zeros(rows * cols, dtype=torch.float32, device="cuda")
        perf.perf_softmax_variant(xd.data_ptr(), yd.data_ptr(), rows, cols, cols, cols, perf.PERF_F32, perf.PERF_F32, 1.0,
                                  rpw, wpr, grid, G.stream())
        torch.cuda.synchronize()
        P.assert_softmax_close(yd.cpu().numpy().reshape(rows, cols), ref)
        ran += 1
    for wpr, rpw in [(1, 8), (1, 3), (4, 2), (2, 0)]:        # too many registers; not a power of two; knob of another family; no such family
        rc = perf.perf_softmax_variant(xd.data_ptr(), xd.data_ptr(), rows, cols, cols, cols, perf.PERF_F32, perf.PERF_F32,
                                       1.0, rpw, wpr, 0, G.stream(), check=False)
        assert rc == perf.PERF_ERR_UNSUPPORTED, (wpr, rpw)
    d = configs.LayerNormWorkload(rows=200, cols=2048).make()
    refy, mref, rref = oracle.layernorm(oracle.widen(d["x_bf16"], True), d["gamma"], d["beta"], float(np.float32(1e-5)))
    xd, gd, bd = G.dev(d["x_bf16"]), G.dev(d["gamma"]), G.dev(d["beta"])
    for wpr, grid in [(1, 0), (1, 10), (4, 0), (4, 3), (16, 0), (16, 2), (0, 40)]:
        yd = torch.zeros(200 * 2048, dtype=torch.float32, device="cuda")
        md, rd = torch.zeros(200, device="cuda"), torch.zeros(200, device="cuda")
        perf.perf_layernorm_variant(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), yd.data_ptr(), md.data_ptr(), rd.data_ptr(),
                                    200, 2048, 2048, 2048, 1e-5, perf.PERF_BF16, perf.PERF_F32, perf.PERF_F32, wpr, grid,
                                    G.stream())
        torch.cuda.synchronize()
        y = yd.cpu().numpy().reshape(200, 2048).astype(np.float64)
        rms = np.sqrt((refy ** 2).mean(axis=1, keepdims=True))
        assert np.max(np.abs(y - refy) / np.maximum(np.abs(refy), rms)) <= 1e-5, (wpr, grid)
        assert np.max(np.abs(rd.cpu().numpy() - rref) / rref) <= 1e-5
    rc = perf.perf_layernorm_variant(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), xd.data_ptr(), None, None, 200, 2048, 2048,
                                     2048, 1e-5, perf.PERF_BF16, perf.PERF_F32, perf.PERF_BF16, 2, 0, G.stream(), check=False)
    assert rc == perf.PERF_ERR_UNSUPPORTED


def test_search_reductions_all_points_and_annealing_walk():
    out = tune.search_softmax(4096, 512, iters=2, warmup=1, strategy="random", budget=1)     # (its seeded input)

    def against_oracle(o, ref=oracle.softmax(out["inputs"]["x"])):
        rel, small = P.softmax_max_rel_err(o, ref)
        return rel <= 1e-5 and small <= 1e-35, rel
    out = tune.search_softmax(4096, 512, iters=5, warmup=2, validate=against_oracle)
    ok = [r for r in out["results"] if r["status"] == "ok"]
    # 512 columns: 2 vectors per lane, so 1, 2, 4 or 8 rows per wave; 4 or 16 waves per row; 5 grids each
    assert len(ok) == (4 + 2) * 5 and not any(r["status"] == "rejected" for r in out["results"])
    assert out["default_us"] <= out["best"]["us"] * 1.5
    walk = tune.search_layernorm(2048, 4096, iters=5, warmup=2, strategy="anneal", budget=12, seed=1)
    assert walk["best"] is not None and 2 <= walk["visited"] <= 13
    full = tune.search_layernorm(2048, 4096, iters=5, warmup=2)
    assert full["visited"] == 18 and full["best"]["us"] <= walk["best"]["us"] * 1.5
