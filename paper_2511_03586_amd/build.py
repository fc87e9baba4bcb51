"""Build libperf.so (the C-ABI operator library) for gfx950 with hipcc.

Usage: ``python -m paper_2511_03586_amd.build``. hipcc cross-compiles, so this works on a
machine without a GPU. Objects go to ``_build/`` (ignored); the library is written next to
this file, where the binding looks for it.

``python -m paper_2511_03586_amd.build --timeline`` builds, beside it, the two diagnostic
libraries ``libperf_timeline1.so`` / ``libperf_timeline2.so``: the same sources with the
cycle-counter stamps of ``csrc/timeline.h`` compiled in (phase stamps / plus one stamp per
main-loop step). ``paper_2511_03586_amd.timeline`` runs them; nothing else loads them.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libperf.so")
SOURCES = ["misc.hip", "softmax.hip", "layernorm.hip", "gemm.hip", "gemm_softmax.hip", "conv2d.hip", "streaming.hip", "batchnorm.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
         # keep the compiler from forming packed-fp32 VALU ops
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _compile(src: str, objdir: str, defines=()) -> str:
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(lambda s: _compile(s, objdir), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose:
        print(f"built {LIB}")
    return LIB


def timeline_lib(level: int) -> str:
    return os.path.join(HERE, f"libperf_timeline{level}.so")


def build_timeline(verbose: bool = True) -> None:
    for level in (1, 2):
        objdir = os.path.join(HERE, "_build", f"timeline{level}")
        os.makedirs(objdir, exist_ok=True)
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            objs = list(pool.map(lambda s: _compile(s, objdir, (f"-DPERF_TIMELINE={level}",)), SOURCES))
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", timeline_lib(level), *objs])
        if verbose:
            print(f"built {timeline_lib(level)}")


if __name__ == "__main__":
    if "--timeline" in sys.argv[1:]:
        build_timeline()
    else:
        build()
