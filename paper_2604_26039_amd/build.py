"""Builds libramp.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2604_26039_amd.build [--force]

Objects are compiled in parallel and cached by source mtime under _build/ (not committed);
hipcc cross-compiles without a GPU.

The kernel translation units are compiled with -Rpass-analysis=kernel-resource-usage; the registers,
LDS bytes and wavefronts per SIMD that the compiler reports for every projection kernel go into
_build/kernel_resources.inc, which resources.cpp compiles into the library: the cost model's wave
capacity W(c) comes from that table.
"""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libramp.so")
OBJ_DIR = os.path.join(PKG, "_build")

KERNEL_SOURCES = ["gemm_group0.hip", "gemm_group1.hip", "gemm_group2.hip", "gemm_group3.hip", "gemm_group4.hip",
                  "gemm_group5.hip", "gemm_group6.hip", "gemm_group7.hip", "stream_group0.hip", "stream_group1.hip",
                  "stream_group2.hip"]
SOURCES = ["align.hip", "select.hip", "pack.hip", "fused.hip", "fp8.hip"] + KERNEL_SOURCES + ["cost_model.cpp"]
HEADERS = ["ramp_internal.h", "moe_gemm.h", "moe_pingpong.h", "moe_stream.h", "moe_decode.h", "align_tiny.h", "config_list.h", os.path.join(ROOT, "include", "ramp.h")]

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-ffp-contract=off"]
# packed fp32 ops are disabled on purpose: some of their forms have produced wrong results on this hardware
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]
FAMILIES = ("moe_gemm_kernel", "moe_pingpong_kernel", "moe_stream_kernel")


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


def _parse_resources(stderr: str) -> list:
    """[{family, targs, vgprs, agprs, lds, waves_per_simd}] from hipcc's kernel-resource-usage remarks."""
    out, cur = [], None
    for line in stderr.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = None
            name = m.group(1)
            fam = next((f for f in FAMILIES if f"{len(f)}{f}I" in name), None)
            if fam is None:
                continue
            args = name.split(f"{len(fam)}{fam}I", 1)[1]
            targs = [int(v) for v in re.findall(r"Li(\d+)E", args.split("EEv", 1)[0] + "E")]
            cur = dict(family=fam, targs=targs)
            out.append(cur)
            continue
        if cur is None:
            continue
        for key, pat in (("vgprs", r"remark:\s+VGPRs: (\d+)"), ("agprs", r"remark:\s+AGPRs: (\d+)"),
                         ("waves_per_simd", r"remark:\s+Occupancy \[waves/SIMD\]: (\d+)"),
                         ("lds", r"remark:\s+LDS Size \[bytes/block\]: (\d+)")):
            m = re.search(pat, line)
            if m:
                cur[key] = int(m.group(1))
    return out


def _compile(src: str, force: bool, hdr_time: float) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(OBJ_DIR, src + ".o")
    res_json = os.path.join(OBJ_DIR, src + ".resources.json")
    is_kernel = src in KERNEL_SOURCES
    if (not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), hdr_time)
            and (not is_kernel or os.path.exists(res_json))):
        return obj
    cmd = [_hipcc()] + COMMON
    if src.endswith(".hip"):
        cmd += HIP_FLAGS
        if is_kernel:
            cmd += ["-Rpass-analysis=kernel-resource-usage"]
    else:
        cmd += ["-x", "c++"]
    cmd += ["-c", path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    if is_kernel:
        entries = _parse_resources(res.stderr)
        if not entries or any(len({"vgprs", "agprs", "lds", "waves_per_simd"} - set(e)) for e in entries):
            raise RuntimeError(f"{src}: could not read the compiler's kernel resource usage")
        with open(res_json, "w") as f:
            json.dump(entries, f)
    return obj


def _resource_table() -> str:
    """Writes _build/kernel_resources.inc from the per-source resource records; returns its path."""
    lines = []
    for src in KERNEL_SOURCES:
        with open(os.path.join(OBJ_DIR, src + ".resources.json")) as f:
            for e in json.load(f):
                targs = list(e["targs"]) + [0] * (8 - len(e["targs"]))
                lines.append('    {"%s", %d, {%s}, %d, %d, %d, %d},' % (e["family"], len(e["targs"]), ", ".join(map(str, targs)),
                                                                      e["vgprs"], e["agprs"], e["lds"], e["waves_per_simd"]))
    path = os.path.join(OBJ_DIR, "kernel_resources.inc")
    text = "\n".join(sorted(set(lines))) + "\n"
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
    return path


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = _newest_header()
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force, hdr_time), SOURCES))
    inc = _resource_table()
    res_obj = os.path.join(OBJ_DIR, "resources.cpp.o")
    res_src = os.path.join(CSRC, "resources.cpp")
    if force or not os.path.exists(res_obj) or os.path.getmtime(res_obj) < max(os.path.getmtime(inc), os.path.getmtime(res_src), hdr_time):
        cmd = [_hipcc()] + COMMON + HIP_FLAGS + ["-I", OBJ_DIR, "-x", "hip", "-c", res_src, "-o", res_obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    objs.append(res_obj)
    if force or not os.path.exists(OUT) or any(os.path.getmtime(o) > os.path.getmtime(OUT) for o in objs):
        cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT] + objs
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"link failed: {' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    return OUT


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
