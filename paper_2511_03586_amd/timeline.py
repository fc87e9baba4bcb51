"""Cycle-counter timelines of the GEMM and convolution kernels (diagnostic builds).

``python -m paper_2511_03586_amd.build --timeline`` builds ``libperf_timeline1.so`` (phase
stamps only) and ``libperf_timeline2.so`` (plus one stamp per main-loop step) from the same
sources as the product library with ``csrc/timeline.h`` switched on; this module launches
the 4096^3 GEMM and the 3x3 64 -> 128 convolution through them, with random and with zero
operands, and prints where the cycles of a workgroup go (median over the 256 workgroups of
the last launch) together with the shader clock the kernel ran at (cycle counter against
the constant 100 MHz clock).  Usage, on a GPU machine::

    python -m paper_2511_03586_amd.timeline            # markdown on stdout

Inputs are the bench workloads' recipes (uniform[0,1) activations, N(0, 2/fan-in) weights;
uniform[-1,1) GEMM operands), drawn with torch on the device: the values do not matter
here, only whether they toggle the datapath (random) or not (zeros).
"""
from __future__ import annotations

import ctypes
import sys

import numpy as np

from .build import timeline_lib

GROUPS, ROLES, SLOTS = 256, 2, 64
i64, ptr, cint, f32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float


def _load(path):
    lib = ctypes.CDLL(path)
    lib.perf_conv2d_variant.restype = cint
    lib.perf_conv2d_variant.argtypes = [ptr, ptr, ptr] + [i64] * 11 + [cint, cint, cint, ptr]
    lib.perf_gemm.restype = cint
    lib.perf_gemm.argtypes = [ptr, ptr, ptr, i64, i64, i64, cint, i64, cint, i64, i64, i64, i64, i64, i64, f32, cint, cint, ptr]
    for name in ("perf_timeline_fetch_conv", "perf_timeline_fetch_gemm"):
        getattr(lib, name).restype = cint
        getattr(lib, name).argtypes = [ptr]
    return lib


def _fetch(fn):
    out = np.zeros((GROUPS, ROLES, SLOTS), dtype=np.int64)
    rc = fn(out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"timeline fetch failed ({rc})")
    return out


def _med(a):
    a = a[a > 0]
    return int(np.median(a)) if a.size else 0


def _clock(buf, role):
    cyc, ticks = buf[:, role, 0].astype(np.float64), buf[:, role, 1].astype(np.float64)
    ok = ticks > 0
    return float(np.median(cyc[ok] / (ticks[ok] * 10.0)))  # GHz: cycles per ns, one tick = 10 ns


def conv_timeline(torch, lib, variant, zeros, launches=24):
    N, H, W, C, K = 32, 56, 56, 64, 128
    st = torch.cuda.current_stream().cuda_stream
    if zeros:
        x = torch.zeros(4, N, H, W, C, device="cuda", dtype=torch.bfloat16)
        w = torch.zeros(K, 3, 3, C, device="cuda", dtype=torch.bfloat16)
    else:
        x = torch.rand(4, N, H, W, C, device="cuda").to(torch.bfloat16)
        w = (torch.randn(K, 3, 3, C, device="cuda") * (2.0 / 576) ** 0.5).to(torch.bfloat16)
    y = torch.empty(4, N, H, W, K, device="cuda", dtype=torch.bfloat16)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(launches):
        if i == launches // 2:
            e0.record()
        rc = lib.perf_conv2d_variant(x[i % 4].data_ptr(), w.data_ptr(), y[i % 4].data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 1, 1,
                                     1, 1, variant, st)
        if rc != 0:
            raise RuntimeError(f"perf_conv2d_variant({variant}) returned {rc}")
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1000 / (launches - launches // 2)
    return _fetch(lib.perf_timeline_fetch_conv), us


def gemm_timeline(torch, lib, zeros, launches=8):
    n = 4096
    st = torch.cuda.current_stream().cuda_stream
    if zeros:
        a = torch.zeros(2, n, n, device="cuda", dtype=torch.bfloat16)
        b = torch.zeros(2, n, n, device="cuda", dtype=torch.bfloat16)
    else:
        a = (torch.rand(2, n, n, device="cuda") * 2 - 1).to(torch.bfloat16)
        b = (torch.rand(2, n, n, device="cuda") * 2 - 1).to(torch.bfloat16)
    c = torch.empty(2, n, n, device="cuda", dtype=torch.float32)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(launches):
        if i == launches // 2:
            e0.record()
        # row-major A x column-major B, bf16 in, fp32 out
        rc = lib.perf_gemm(a[i % 2].data_ptr(), b[i % 2].data_ptr(), c[i % 2].data_ptr(), n, n, n, 0, n, 1, n, n, 1, 0, 0, 0,
                           1.0, 1, 0, st)
        if rc != 0:
            raise RuntimeError(f"perf_gemm returned {rc}")
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1000 / (launches - launches // 2)
    return _fetch(lib.perf_timeline_fetch_gemm), us


def main():
    import torch
    if not torch.cuda.is_available():
        sys.exit("timeline: needs a GPU")
    l1, l2 = _load(timeline_lib(1)), _load(timeline_lib(2))
    print("## GEMM 4096^3 bf16 -> fp32 (`gemm_mfma_kernel<4,4,2,2,K64,f32>`, 256 workgroups, one per CU)\n")
    print("Wave 0 of each workgroup, cycles since the workgroup started, median over workgroups (phase stamps only).\n")
    print("| operands | us / launch (events) | clock GHz | main loop begins | main loop ends | loop cycles | loop us | "
          "MFMA minimum 131 072 cycles = % of loop | stores issued | stores complete |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for zeros in (False, True):
        buf, us = gemm_timeline(torch, l1, zeros)
        ghz = _clock(buf, 0)
        t2, t3, t4, t0 = (_med(buf[:, 0, s]) for s in (2, 3, 4, 0))
        loop = t3 - t2
        print(f"| {'zeros' if zeros else 'uniform[-1,1)'} | {us:.1f} | {ghz:.2f} | {t2} | {t3} | {loop} | {loop / ghz / 1e3:.1f} | "
              f"{100.0 * 131072 / loop:.0f} | {t4} | {t0} |")
    print()
    names = {6: "`conv2d_wres_kernel<3,3,64,bf16>` (128 channels per workgroup, input rows resident)",
             8: "`conv2d_wsplit_kernel<3,3,64,bf16>` (64-channel slabs, input-row ring; the library's choice)"}
    for variant in (8, 6):
        print(f"## conv 32x56x56x64 -> 128, 3x3, bf16: {names[variant]}, 256 workgroups\n")
        print("MFMA wave 0 and memory wave 4 of each workgroup, cycles since the workgroup started, median over workgroups. "
              "Phase stamps only (the steady-state figure is undisturbed):\n")
        if variant == 6:
            print("| operands | us / launch (events) | clock GHz | first rows issued (memory wave) | first rows landed | weights in "
                  "registers (MFMA wave) | first MFMA (after barrier) | last block done | end | blocks | cycles per block | "
                  "MFMA minimum 1152 = % |")
            print("|---|---|---|---|---|---|---|---|---|---|---|---|")
        else:
            print("| operands | us / launch (events) | clock GHz | first rows issued (memory wave) | first rows landed | weights and "
                  "rows complete, first MFMA | steps 0 and 1 done | last step done | end | steps after the first two | "
                  "cycles per step | MFMA minimum 1152 = % |")
            print("|---|---|---|---|---|---|---|---|---|---|---|---|")
        for zeros in (False, True):
            buf, us = conv_timeline(torch, l1, variant, zeros)
            ghz = _clock(buf, 0)
            m = lambda role, s: _med(buf[:, role, s])
            if variant == 6:
                steps = 13
                per = (m(0, 4) - m(0, 3)) / steps
                print(f"| {'zeros' if zeros else 'random'} | {us:.2f} | {ghz:.2f} | {m(1, 2)} | {m(1, 3)} | {m(0, 2)} | {m(0, 3)} | "
                      f"{m(0, 4)} | {m(0, 0)} | {steps} | {per:.0f} | {100 * 1152 / per:.0f} |")
            else:
                steps = 11
                per = (m(0, 6) - m(0, 5)) / steps
                print(f"| {'zeros' if zeros else 'random'} | {us:.2f} | {ghz:.2f} | {m(1, 2)} | {m(1, 3)} | {m(0, 4)} | {m(0, 5)} | "
                      f"{m(0, 6)} | {m(0, 0)} | {steps} | {per:.0f} | {100 * 1152 / per:.0f} |")
        buf, us = conv_timeline(torch, l2, variant, False)
        first = 0 if variant == 6 else 2
        tops = [_med(buf[:, 0, 8 + t]) for t in range(first, 13)]
        mem = [_med(buf[:, 1, 8 + t]) for t in range(first, 13)]
        print(f"\nWith a stamp per step (random operands, {us:.2f} us / launch: every stamp drains the wave's LDS reads once), "
              "MFMA wave at the top of each step / memory wave behind the step's barrier:\n")
        print("| step | " + " | ".join(str(t) for t in range(first, 13)) + " |")
        print("|---|" + "---|" * len(tops))
        print("| MFMA wave | " + " | ".join(str(v) for v in tops) + " |")
        print("| memory wave | " + " | ".join(str(v) for v in mem) + " |")
        print()


if __name__ == "__main__":
    main()
