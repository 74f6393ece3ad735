"""Build step: compiles the HIP sources in csrc/ into libsagnn.so for gfx950 (in-tree)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB = os.path.join(_HERE, "libsagnn.so")
OBJDIR = os.path.join(_HERE, "_build")
SOURCES = ["api.hip", "pack.hip", "plan.hip", "spmm.hip", "spmm_sweep.hip", "gemm.hip", "stages.hip",
           "fused.hip", "permute.hip", "sweep_plan.hip", "tiles.hip"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(CSRC, "rowload.h"), os.path.join(INCLUDE, "sagnn.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed fp32 VALU ops are kept off (plain v_fma_f32 only)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-pass-failed",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + HEADERS)


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))


def build_hip(verbose: bool = False, incremental: bool = False, jobs: int = 8) -> str:
    """Compile every source to an object file (in parallel) and link libsagnn.so.  With
    incremental=True only sources newer than their object file are recompiled."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    hdr_t = max(os.path.getmtime(h) for h in HEADERS)
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_t))
        if not fresh:
            todo.append([hipcc, *HIPCC_FLAGS, f"-I{INCLUDE}", "-c", "-o", obj, src])
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        list(ex.map(lambda c: _run(c, verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB
