"""Timing-driven choice among the library's kernel variants: the one piece of the paper's
search loop that a fixed kernel library can show (Section 3: a candidate program is emitted,
its output is validated against the untransformed program, and it is scored by its measured
runtime, reward c / T; Section 4.2: warm-up runs, then timed runs on fresh input data).

A search space is a set of axes (name -> values); a point picks one value per axis.  Three ways
of visiting it, the paper's classical baselines (Section 4.2): every point (`strategy="all"`),
a random sample (`"random"`), or a simulated-annealing walk whose cost is the candidate's own
runtime (`"anneal"`: a neighbour differs in one axis by one step; a slower neighbour is accepted
with probability exp(-relative slowdown / temperature), the temperature falls geometrically).
Every visited point is first validated: its output on one input set goes through `validate`,
by default a comparison with the output of the library's own choice (the "untransformed
program"); callers may pass any other check, e.g. against an independent reference.

Inputs come from the seeded host generators in `workloads/` and all comparisons are done on the
host with numpy; torch only holds device memory and times the launches.  The transformation
language, its embedding and the learned agent are out of scope.

Usage:  python -m paper_2511_03586_amd.tune gemm M N K [batch] [strategy]
        python -m paper_2511_03586_amd.tune conv N H W C K R S [stride pad] [strategy]
        python -m paper_2511_03586_amd.tune softmax rows cols [strategy]
        python -m paper_2511_03586_amd.tune layernorm rows cols [strategy]
"""
from __future__ import annotations

import itertools
import math
import os
import random
import sys

import numpy as np
import torch

import paper_2511_03586_amd as perf

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from workloads import rng  # noqa: E402  (seeded input generators: no operator arithmetic)

# kstep 33: K-step 32 with the deep ring; 65: K-step 64 built on the 32x32x16 MFMA (256x256 tile only)
GEMM_AXES = {"tile": (64, 128, 256), "kstep": (32, 33, 64, 65)}
CONV_AXES = {"variant": (perf.CONV_WRES, perf.CONV_WREG, perf.CONV_WSPLIT, perf.CONV_MFMA, perf.CONV_F32MFMA, perf.CONV_ROWMFMA,
                         perf.CONV_SMALLC, perf.CONV_DIRECT)}
CONV_NAMES = {perf.CONV_WRES: "weights-in-regs, input-in-lds", perf.CONV_WREG: "weights-in-registers",
              perf.CONV_WSPLIT: "weights-in-regs, 64-channel slabs",
              perf.CONV_MFMA: "implicit-gemm", perf.CONV_F32MFMA: "implicit-gemm-fp32-mfma", perf.CONV_ROWMFMA: "filter-row-per-mfma",
              perf.CONV_SMALLC: "channel-blocked-direct", perf.CONV_DIRECT: "thread-per-output"}
# grid_per_cu: workgroups per CU of a persistent grid; 0 = the kernel family's own default
SOFTMAX_AXES = {"waves_per_row": (1, 4, 16), "rows_per_wave": (0, 1, 2, 4, 8), "grid_per_cu": (0, 2, 4, 8, 16)}
LAYERNORM_AXES = {"waves_per_row": (1, 4, 16), "grid_per_cu": (2, 4, 6, 8, 12, 16)}


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


def _dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def _host(t: torch.Tensor) -> np.ndarray:
    a = t.cpu().numpy()
    if a.dtype == np.int16:  # bf16 bit patterns
        return rng.bf16_bits_to_f32(a.view(np.uint16)).astype(np.float64)
    return a.astype(np.float64)


def max_rel_diff(out: np.ndarray, ref: np.ndarray) -> float:
    """max |out - ref| / max |ref|."""
    return float(np.max(np.abs(out - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def _points(axes):
    names = list(axes)
    return [dict(zip(names, vals)) for vals in itertools.product(*(axes[n] for n in names))]


def _key(point):
    return tuple(sorted(point.items()))


def search(axes, run, validate, work, nsets, iters=30, warmup=5, strategy="all", budget=None, seed=0, t0=0.05,
           cooling=0.8):
    """Visit points of ``axes``.  ``run(point, set) -> device tensor | None`` launches the variant on
    buffer set ``set`` and returns its output (None = the variant cannot run the problem);
    ``validate(host_output) -> (ok, error)``.  Returns {"results": [...], "best": ..., "visited": n}."""
    rnd = random.Random(seed)
    cache = {}

    def evaluate(point):
        k = _key(point)
        if k in cache:
            return cache[k]
        out = run(point, 0)  # also the validation launch
        if out is None:
            res = {"variant": dict(point), "status": "unsupported"}
        else:
            torch.cuda.synchronize()
            ok, err = validate(_host(out))
            if not ok:
                res = {"variant": dict(point), "status": "rejected", "error": err}
            else:
                us = _time(lambda s: run(point, s), nsets, iters, warmup)
                res = {"variant": dict(point), "status": "ok", "us": us, "reward": work / us, "error": err}
        cache[k] = res
        return res

    pts = _points(axes)
    if strategy == "all":
        for p in pts:
            evaluate(p)
    elif strategy == "random":
        for p in rnd.sample(pts, min(budget or len(pts), len(pts))):
            evaluate(p)
    elif strategy == "anneal":
        names = list(axes)
        steps = budget or 2 * sum(len(v) for v in axes.values())
        cur = rnd.choice(pts)
        for _ in range(4 * len(pts)):  # a start the library can run
            if evaluate(cur)["status"] == "ok":
                break
            cur = rnd.choice(pts)
        temp = t0
        for _ in range(steps):
            n = rnd.choice(names)
            i = axes[n].index(cur[n]) + rnd.choice((-1, 1))
            if not 0 <= i < len(axes[n]):
                continue
            nxt = dict(cur, **{n: axes[n][i]})
            a, b = evaluate(cur), evaluate(nxt)
            if b["status"] == "ok" and (a["status"] != "ok" or b["us"] <= a["us"] or
                                        rnd.random() < math.exp(-(b["us"] / a["us"] - 1.0) / temp)):
                cur = nxt
            temp *= cooling
    else:
        raise ValueError(f"unknown strategy {strategy!r}")
    results = list(cache.values())
    ok = [r for r in results if r["status"] == "ok"]
    return {"results": results, "best": min(ok, key=lambda r: r["us"]) if ok else None, "visited": len(results)}


def _against(reference: np.ndarray, tol: float):
    def validate(out):
        err = max_rel_diff(out, reference)
        return err <= tol, err
    return validate


def search_gemm(M, N, K, batch=1, c_f32=True, validate=None, tol=1e-5, **kw):
    """GEMM variants for C = A * B^T-as-stored (bf16 U[-1,1] operands, fp32 accumulate).  Default
    validation: against the output of the library's own choice (the variants share the accumulation
    order per K-step kind), 1e-5 relative to max |C|.  Adds "default_us", "inputs" (the host operands
    of set 0, for callers that validate against their own reference)."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    cdt = perf.PERF_F32 if c_f32 else perf.PERF_BF16
    nsets = _rotating_sets(batch * (M * K + N * K) * 2 + batch * M * N * (4 if c_f32 else 2))
    seed = kw.get("seed", 0)
    a0 = rng.f32_to_bf16_bits(rng.uniform(rng.tensor_seed(3, 0, seed), (batch, M, K), -1.0, 1.0))
    b0 = rng.f32_to_bf16_bits(rng.uniform(rng.tensor_seed(3, 1, seed), (batch, N, K), -1.0, 1.0))
    a = torch.stack([torch.roll(_dev(a0), s, 1) for s in range(nsets)])
    b = torch.stack([torch.roll(_dev(b0), s, 1) for s in range(nsets)])
    c = torch.empty((nsets, batch, M, N), device="cuda", dtype=torch.float32 if c_f32 else torch.int16)
    args = lambda s: (a[s].data_ptr(), b[s].data_ptr(), c[s].data_ptr(), M, N, K, perf.PERF_ROW_MAJOR, K,
                      perf.PERF_COL_MAJOR, K, N, batch, M * K, N * K, M * N, 1.0, perf.PERF_BF16, cdt)

    def default(s):
        perf.perf_gemm(*args(s), st())
        return c[s]

    def run(p, s):
        rc = perf.perf_gemm_variant(*args(s), p["tile"], p["kstep"], st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_gemm_variant", rc)
        return c[s]

    if validate is None:
        reference = _host(default(0))
        validate = _against(reference, tol)
    out = search(GEMM_AXES, run, validate, 2.0 * batch * M * N * K * 1e-6, nsets, **kw)
    out["default_us"] = _time(default, nsets, kw.get("iters", 30), kw.get("warmup", 5))
    out["inputs"] = {"a_bf16": a0, "b_bf16": b0}
    return out


def search_conv(N, H, W, C, K, R, S, stride=1, pad=1, y_bf16=True, validate=None, **kw):
    """Convolution kernel families for NHWC bf16 input U[0,1], KRSC bf16 weights N(0, 2 / (R S C))."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    ydt = perf.PERF_BF16 if y_bf16 else perf.PERF_F32
    nsets = _rotating_sets(N * H * W * C * 2 + N * P * Q * K * (2 if y_bf16 else 4))
    seed = kw.get("seed", 0)
    x0 = rng.f32_to_bf16_bits(rng.uniform(rng.tensor_seed(5, 0, seed), (N, H, W, C), 0.0, 1.0))
    w0 = rng.f32_to_bf16_bits(rng.normal(rng.tensor_seed(5, 1, seed), (K, R, S, C), 0.0, 2.0 / (R * S * C)))
    x = torch.stack([torch.roll(_dev(x0), s, 1) for s in range(nsets)])
    w = _dev(w0)
    y = torch.empty((nsets, N, P, Q, K), device="cuda", dtype=torch.int16 if y_bf16 else torch.float32)
    args = lambda s: (x[s].data_ptr(), w.data_ptr(), y[s].data_ptr(), N, H, W, C, K, R, S, stride, stride, pad, pad,
                      perf.PERF_BF16, ydt)

    def default(s):
        perf.perf_conv2d(*args(s), st())
        return y[s]

    def run(p, s):
        rc = perf.perf_conv2d_variant(*args(s), p["variant"], st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_conv2d_variant", rc)
        return y[s]

    if validate is None:
        # different kernels sum in different orders, and bf16 outputs differ by one rounding
        validate = _against(_host(default(0)), 2.0 ** -7 if y_bf16 else 1e-4)
    out = search(CONV_AXES, run, validate, 2.0 * N * P * Q * K * R * S * C * 1e-6, nsets, **kw)
    out["default_us"] = _time(default, nsets, kw.get("iters", 30), kw.get("warmup", 5))
    out["inputs"] = {"x_bf16": x0, "w_bf16": w0}
    return out


def search_softmax(rows, cols, validate=None, tol=2e-6, **kw):
    """Launch shapes of the row softmax (fp32, entries N(0, 4)): rows per wave, waves per row, grid.
    Default validation: against the library's own choice; the variants differ only in the summation
    tree of the row sum, so 2e-6 relative to the largest probability."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    nsets = _rotating_sets(8 * rows * cols)
    x0 = rng.normal(rng.tensor_seed(1, 0, kw.get("seed", 0)), (rows, cols), 0.0, 4.0)
    x = torch.stack([torch.roll(_dev(x0), s, 0) for s in range(nsets)])
    y = torch.empty_like(x)
    F32 = perf.PERF_F32

    def default(s):
        perf.perf_softmax(x[s].data_ptr(), y[s].data_ptr(), rows, cols, cols, cols, F32, F32, 1.0, st())
        return y[s]

    def run(p, s):
        wpr, rpw, g = p["waves_per_row"], p["rows_per_wave"], p["grid_per_cu"]
        if (wpr == 1) != (rpw != 0):
            return None  # rows per wave is a knob of the wave-per-row kernels only
        rc = perf.perf_softmax_variant(x[s].data_ptr(), y[s].data_ptr(), rows, cols, cols, cols, F32, F32, 1.0, rpw, wpr,
                                       256 * g, st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_softmax_variant", rc)
        return y[s]

    if validate is None:
        validate = _against(_host(default(0)), tol)
    out = search(SOFTMAX_AXES, run, validate, 8.0 * rows * cols * 1e-6, nsets, **kw)
    out["default_us"] = _time(default, nsets, kw.get("iters", 30), kw.get("warmup", 5))
    out["inputs"] = {"x": x0}
    return out


def search_layernorm(rows, cols, bf16=True, validate=None, **kw):
    """Launch shapes of LayerNorm (x ~ N(1, 3), gamma ~ U[0.5, 1.5], beta ~ N(0, 0.1); bf16 or fp32 in
    and out): waves per row, workgroups per CU.  Default validation against the library's own choice:
    one bf16 rounding apart at most (2^-7 relative to the largest output), 1e-5 for fp32."""
    st = lambda: torch.cuda.current_stream().cuda_stream
    esz = 2 if bf16 else 4
    nsets = _rotating_sets(2 * esz * rows * cols)
    seed = kw.get("seed", 0)
    xf = rng.normal(rng.tensor_seed(2, 0, seed), (rows, cols), 1.0, 3.0)
    x0 = rng.f32_to_bf16_bits(xf) if bf16 else xf
    g0 = rng.uniform(rng.tensor_seed(2, 1, seed), (cols,), 0.5, 1.5)
    b0 = rng.normal(rng.tensor_seed(2, 2, seed), (cols,), 0.0, 0.1)
    x = torch.stack([torch.roll(_dev(x0), s, 0) for s in range(nsets)])
    y = torch.empty_like(x)
    g, b = _dev(g0), _dev(b0)
    dt = perf.PERF_BF16 if bf16 else perf.PERF_F32
    args = lambda s: (x[s].data_ptr(), g.data_ptr(), b.data_ptr(), y[s].data_ptr(), None, None, rows, cols, cols, cols,
                      1e-5, dt, perf.PERF_F32, dt)

    def default(s):
        perf.perf_layernorm(*args(s), st())
        return y[s]

    def run(p, s):
        rc = perf.perf_layernorm_variant(*args(s), p["waves_per_row"], 256 * p["grid_per_cu"], st(), check=False)
        if rc == perf.PERF_ERR_UNSUPPORTED:
            return None
        if rc != perf.PERF_OK:
            raise perf.PerfError("perf_layernorm_variant", rc)
        return y[s]

    if validate is None:
        validate = _against(_host(default(0)), 2.0 ** -7 if bf16 else 1e-5)
    out = search(LAYERNORM_AXES, run, validate, 2.0 * esz * rows * cols * 1e-6, nsets, **kw)
    out["default_us"] = _time(default, nsets, kw.get("iters", 30), kw.get("warmup", 5))
    out["inputs"] = {"x": x0, "gamma": g0, "beta": b0}
    return out


def _print(kind, out, name=lambda v: str(v)):
    for r in sorted(out["results"], key=lambda r: r.get("us", float("inf"))):
        if r["status"] == "ok":
            print(f"  {name(r['variant']):44s} {r['us']:10.2f} us   reward {r['reward']:12.1f} /us   error {r['error']:.1e}")
        elif r["status"] == "rejected":
            print(f"  {name(r['variant']):44s} rejected (error {r['error']:.1e})")
    b = out["best"]
    n_unsup = sum(r["status"] == "unsupported" for r in out["results"])
    if b is None:
        print(f"{kind}: no variant ran ({n_unsup} unsupported)")
    else:
        print(f"{kind}: visited {out['visited']} points ({n_unsup} cannot run this problem); best {name(b['variant'])} "
              f"at {b['us']:.2f} us; the library's own choice takes {out['default_us']:.2f} us")


def main(argv):
    strategy = argv.pop() if argv and argv[-1] in ("all", "random", "anneal") else "all"
    kw = {"strategy": strategy}
    if len(argv) >= 4 and argv[0] == "gemm":
        M, N, K = (int(v) for v in argv[1:4])
        batch = int(argv[4]) if len(argv) > 4 else 1
        _print("gemm", search_gemm(M, N, K, batch, **kw))
    elif len(argv) >= 8 and argv[0] == "conv":
        N, H, W, C, K, R, S = (int(v) for v in argv[1:8])
        stride = int(argv[8]) if len(argv) > 8 else 1
        pad = int(argv[9]) if len(argv) > 9 else R // 2
        _print("conv", search_conv(N, H, W, C, K, R, S, stride, pad, **kw), lambda v: CONV_NAMES[v["variant"]])
    elif len(argv) >= 3 and argv[0] == "softmax":
        _print("softmax", search_softmax(int(argv[1]), int(argv[2]), **kw))
    elif len(argv) >= 3 and argv[0] == "layernorm":
        _print("layernorm", search_layernorm(int(argv[1]), int(argv[2]), **kw))
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
