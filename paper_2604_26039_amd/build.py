"""Builds libramp.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2604_26039_amd.build [--force]

Objects are compiled in parallel and cached by source mtime under _build/ (not committed);
hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libramp.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ["align.hip", "select.hip", "pack.hip", "fused.hip", "gemm_group0.hip", "gemm_group1.hip", "gemm_group2.hip",
           "gemm_group3.hip", "gemm_group4.hip", "gemm_group5.hip", "gemm_group6.hip", "gemm_group7.hip", "stream_group0.hip", "stream_group1.hip", "stream_group2.hip", "cost_model.cpp"]
HEADERS = ["ramp_internal.h", "moe_gemm.h", "moe_pingpong.h", "moe_stream.h", "config_list.h", os.path.join(ROOT, "include", "ramp.h")]

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-ffp-contract=off"]
# packed fp32 ops are disabled on purpose: some of their forms have produced wrong results on this hardware
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _newest_header() -> float:
    t = 0.0
    for h in HEADERS:
        p = h if os.path.isabs(h) else os.path.join(CSRC, h)
        t = max(t, os.path.getmtime(p))
    return max(t, os.path.getmtime(os.path.abspath(__file__)))


def _compile(src: str, force: bool, hdr_time: float) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(OBJ_DIR, src + ".o")
    if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), hdr_time):
        return obj
    cmd = [_hipcc()] + COMMON
    if src.endswith(".hip"):
        cmd += HIP_FLAGS
    else:
        cmd += ["-x", "c++"]
    cmd += ["-c", path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = _newest_header()
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force, hdr_time), SOURCES))
    if force or not os.path.exists(OUT) or any(os.path.getmtime(o) > os.path.getmtime(OUT) for o in objs):
        cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT] + objs
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"link failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    return OUT


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
