"""Timing-driven choice among the library's kernel variants: the one piece of the paper's
search loop that a fixed kernel library can show (Section 3: a candidate program is emitted,
its output is validated against the untransformed program, and it is scored by its measured
runtime, reward c / T; Section 4.2: warm-up runs, then timed runs on fresh input data).

The search space here is small (the tile and main-loop variants of the GEMM, the kernel
families of the convolution), so every point is visited; ``sample`` visits a random subset
in the spirit of the paper's random-sampling baseline (Section 4.1). The transformation
language, its embedding and the learned agent are out of scope.

Usage:  python -m paper_2511_03586_amd.tune gemm M N K [batch]
        python -m paper_2511_03586_amd.tune conv N H W C K R S [stride pad]
"""
from __future__ import annotations

import random
import sys

import torch

import paper_2511_03586_amd as perf

# 33: K-step 32 with the deep ring; 65: K-step 64 built on the 32x32x16 MFMA (256x256 tile only)
GEMM_SPACE = [(tile, kstep) for tile in (64, 128, 256) for kstep in (32, 64)] + [(64, 33), (128, 33), (256, 65)]
CONV_SPACE = [perf.CONV_WRES, perf.CONV_WREG, perf.CONV_MFMA, perf.CONV_ROWMFMA, perf.CONV_SMALLC, perf.CONV_DIRECT]
CONV_NAMES = {perf.CONV_WRES: "weights-in-regs, input-in-lds", perf.CONV_WREG: "weights-in-registers", perf.CONV_MFMA: "implicit-gemm", perf.CONV_ROWMFMA: "filter-row-per-mfma",
              perf.CONV_SMALLC: "channel-blocked-direct", perf.CONV_DIRECT: "thread-per-output"}


def _time(launch, nsets, iters, warmup):
    """Mean microseconds per launch over ``iters`` launches on rotated buffer sets."""
    for i in range(warmup):
        launch(i % nsets)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        launch((warmup + i) % nsets)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def _rotating_sets(bytes_per_set, at_least=2, budget=512 << 20):
    return max(at_least, min(16, budget // max(1, bytes_per_set)))


def _search(space, run, reference, work, nsets, iters, warmup, tol, sample, seed):
    points = list(space)
    if sample is not None and sample < len(points):
        points = random.Random(seed).sample(points, sample)
    results = []
    for p in points:
        out = run(p, 0)                      # also the validation launch
        if out is None:
            results.append({"variant": p, "status": "unsupported"})
            continue
        torch.cuda.synchronize()
        err = float((out.float() - reference.float()).abs().max() / reference.float().abs().max().clamp_min(1e-30))
        if not err <= tol:
            results.append({"variant": p, "status": "rejected", "max_rel_diff": err})
            continue
        us = _time(lambda s: run(p, s), nsets, iters, warmup)
        results.append({"variant": p, "status": "ok", "us": us, "reward": work / us, "max_rel_diff": err})
    ok = [r for r in results if r["status"] == "ok"]
    best = min(ok, key=lambda r: r["us"]) if ok else None
    return {"results": results, "best": best}


def search_gemm(M, N, K, batch=1, c_f32=True, iters=30, warmup=5, sample=None, seed=0):
    """Visit the GEMM variants for C = A * B^T-as-stored (bf16, fp32 accumulate). The library's
    own choice (perf_gemm) is the reference program: every variant is validated against its
    output (they share the accumulation order per K-step kind; 1e-5 relative to max|C|) and
    timed on rotated inputs. Returns {"results": [...], "best": ..., "default_us": ...}."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    cdt = perf.PERF_F32 if c_f32 else perf.PERF_BF16
    nsets = _rotating_sets(batch * (M * K + N * K) * 2 + batch * M * N * (4 if c_f32 else 2))
    g = torch.Generator(device="cuda").manual_seed(seed)
    a = (torch.rand((nsets, batch, M, K), device="cuda", generator=g) * 2 - 1).to(torch.bfloat16)
    b = (torch.rand((nsets, batch, N, K), device="cuda", generator=g) * 2 - 1).to(torch.bfloat16)
    c = torch.empty((nsets, batch, M, N), device="cuda", dtype=torch.float32 if c_f32 else torch.bfloat16)
    args = lambda s: (a[s].data_ptr(), b[s].data_ptr(), c[s].data_ptr(), M, N, K, perf.PERF_ROW_MAJOR, K,
                      perf.PERF_COL_MAJOR, K, N, batch, M * K, N * K, M * N, 1.0, perf.PERF_BF16, cdt)

    def default(s):
        perf.perf_gemm(*args(s), st())
        return c[s]

    def run(p, s):
        rc = perf.perf_gemm_variant(*args(s), p[0], p[1], st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_gemm_variant", rc)
        return c[s]

    reference = default(0).clone()
    out = _search(GEMM_SPACE, run, reference, 2.0 * batch * M * N * K * 1e-6, nsets, iters, warmup, 1e-5, sample, seed)
    out["default_us"] = _time(default, nsets, iters, warmup)
    return out


def search_conv(N, H, W, C, K, R, S, stride=1, pad=1, y_bf16=True, iters=30, warmup=5, sample=None, seed=0):
    """Visit the convolution kernel families for NHWC bf16 input, KRSC bf16 weights."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    ydt = perf.PERF_BF16 if y_bf16 else perf.PERF_F32
    nsets = _rotating_sets(N * H * W * C * 2 + N * P * Q * K * (2 if y_bf16 else 4))
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.rand((nsets, N, H, W, C), device="cuda", generator=g).to(torch.bfloat16)
    w = (torch.randn((K, R, S, C), device="cuda", generator=g) * (2.0 / (R * S * C)) ** 0.5).to(torch.bfloat16)
    y = torch.empty((nsets, N, P, Q, K), device="cuda", dtype=torch.bfloat16 if y_bf16 else torch.float32)
    args = lambda s: (x[s].data_ptr(), w.data_ptr(), y[s].data_ptr(), N, H, W, C, K, R, S, stride, stride, pad, pad,
                      perf.PERF_BF16, ydt)

    def default(s):
        perf.perf_conv2d(*args(s), st())
        return y[s]

    def run(p, s):
        rc = perf.perf_conv2d_variant(*args(s), p, st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_conv2d_variant", rc)
        return y[s]

    reference = default(0).clone()
    # different kernels sum in different orders, and bf16 outputs differ by one rounding
    tol = 2.0 ** -7 if y_bf16 else 1e-4
    out = _search(CONV_SPACE, run, reference, 2.0 * N * P * Q * K * R * S * C * 1e-6, nsets, iters, warmup, tol, sample, seed)
    out["default_us"] = _time(default, nsets, iters, warmup)
    return out


def _print(kind, out, name=lambda v: str(v)):
    for r in out["results"]:
        if r["status"] == "ok":
            print(f"  {name(r['variant']):28s} {r['us']:10.2f} us   reward {r['reward']:12.1f} MFLOP/us   max rel diff {r['max_rel_diff']:.1e}")
        else:
            print(f"  {name(r['variant']):28s} {r['status']}")
    b = out["best"]
    print(f"{kind}: best {name(b['variant'])} at {b['us']:.2f} us; the library's own choice takes {out['default_us']:.2f} us")


def main(argv):
    if len(argv) >= 4 and argv[0] == "gemm":
        M, N, K = (int(v) for v in argv[1:4])
        batch = int(argv[4]) if len(argv) > 4 else 1
        _print("gemm", search_gemm(M, N, K, batch), lambda v: f"tile {v[0]} kstep {v[1]}")
    elif len(argv) >= 8 and argv[0] == "conv":
        N, H, W, C, K, R, S = (int(v) for v in argv[1:8])
        stride = int(argv[8]) if len(argv) > 8 else 1
        pad = int(argv[9]) if len(argv) > 9 else R // 2
        _print("conv", search_conv(N, H, W, C, K, R, S, stride, pad), lambda v: CONV_NAMES[v])
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
