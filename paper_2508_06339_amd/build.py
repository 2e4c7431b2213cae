"""Build libsvb.so (HIP, gfx950) in-tree with hipcc.

Usage: python -m paper_2508_06339_amd.build   (or call build_library()).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsvb.so")
SOURCES = ["svb_api.hip", "stage0_prep.hip", "stage1_panel.hip", "stage1_panel_blk.hip", "stage1_fused.hip", "stage1_fused32.hip", "stage1_fused16.hip", "stage2_chase.hip", "stage2_narrow.hip", "stage2_reduce.hip", "stage3_device.hip",
           "stage3_host.cpp"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         # hipcc -O3 forms packed-fp32 instructions by itself; keep them off
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-attributes"]


def _up_to_date(obj: str, src: str) -> bool:
    """Object newer than its source and every header (used only with SVB_BUILD_INCREMENTAL=1)."""
    if not os.path.exists(obj):
        return False
    deps = [src] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "svb.h"))
    return all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps)


def build_library(verbose: bool = True) -> str:
    """Compiles every translation unit (always, unless SVB_BUILD_INCREMENTAL=1 asks to keep the
    objects that are newer than their sources) and links libsvb.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    incremental = os.environ.get("SVB_BUILD_INCREMENTAL", "0") == "1"
    extra = os.environ.get("SVB_EXTRA_HIPCC_FLAGS", "").split()   # e.g. -DSVB_CHASE_TIMING for kernel-phase timing
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        if incremental and not extra and _up_to_date(obj, os.path.join(CSRC, src)):
            continue
        if src.endswith(".cpp"):   # host-only translation unit
            cmd = ["g++", "-O3", "-std=c++17", "-fPIC", "-c", os.path.join(CSRC, src), "-o", obj]
        else:
            cmd = [hipcc, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(f"--- {src}\n{out}", flush=True)
        failed = failed or p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs, "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
    print(LIB)
