"""Builds libsqa.so (the C-ABI library of include/sqa.h) for gfx950 with hipcc,
in-tree, next to this file.  Run as `python -m paper_2404_04793_amd.build`."""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsqa.so")
OBJ_DIR = os.path.join(HERE, "_build")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
# -amdgpu-mfma-vgpr-form keeps MFMA accumulators in ordinary VGPRs: the decode kernel rescales them with
# vector ALU instructions, and with the default (AGPR) form the compiler copied all 32 of them back and
# forth every tile and needed twice the registers.
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-mllvm", "-amdgpu-mfma-vgpr-form", "-Wno-unused-command-line-argument",
             "-Rpass-analysis=kernel-resource-usage"]
HOST_FLAGS = ["-ffp-contract=off"]
# what the compiler reports per kernel (registers, scratch, waves per SIMD), written next to the objects:
# a source change that costs a kernel its occupancy shows up here (and in tests/test_kernel_resources.py)
# before it shows up as a few lost per cent on the GPU
RESOURCES = os.path.join(OBJ_DIR, "kernel_resources.json")
_REMARK = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|"
                     r"Occupancy \[waves/SIMD\]|VGPRs Spill|LDS Size \[bytes/block\]): (\S+)")


def _parse_resources(stderr: str) -> dict:
    out, cur = {}, None
    for key, val in _REMARK.findall(stderr):
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return out


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def sources():
    out = []
    for f in sorted(os.listdir(CSRC)):
        if f.endswith(".hip") or f.endswith(".cpp"):
            out.append(os.path.join(CSRC, f))
    return out


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    cc = _hipcc()

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        flags = HIP_FLAGS if src.endswith(".hip") else HOST_FLAGS
        cmd = [cc] + COMMON + flags + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        res = _parse_resources(r.stderr)
        keep, skip = [], 0
        for l in r.stderr.splitlines():                # drop the resource remarks (and the two source lines
            if "-Rpass-analysis=kernel-resource-usage" in l:   # clang prints under the first of each group)
                skip = 2 if "Function Name" in l else 0
                continue
            if skip and (re.match(r"\s+\d+ \|", l) or re.match(r"\s+\|\s+\^", l)):
                skip -= 1
                continue
            skip = 0
            if "packed-fp32-ops" not in l:
                keep.append(l)
        err = "\n".join(keep)
        if r.returncode != 0:
            raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), err))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj, res

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        done = list(ex.map(compile_one, sources()))
    objs = [o for o, _ in done]
    resources = {}
    for _, res in done:
        resources.update(res)
    with open(RESOURCES, "w") as fh:
        json.dump(resources, fh, indent=0, sort_keys=True)
    cmd = [cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed: %s\n%s" % (" ".join(cmd), r.stderr))
    if verbose:
        print("built", LIB)
    return LIB


def build_microbench(verbose: bool = True) -> str:
    """microbench/store_cost.hip -> _build/store_cost (a standalone executable, not part of libsqa.so):
    the measurement behind the statement that the decode step is bound by what it writes."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    exe = os.path.join(OBJ_DIR, "store_cost")
    cmd = [_hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unused-result",
           os.path.join(HERE, "microbench", "store_cost.hip"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), r.stderr))
    if verbose:
        print("built", exe)
    return exe


def build_demo(verbose: bool = True) -> str:
    """tests/c_abi_demo.cpp -> _build/c_abi_demo: the library used from plain C++ through include/sqa.h
    (needs libsqa.so built; tests/test_gpu_c_abi_demo.py runs it on the GPU)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    exe = os.path.join(OBJ_DIR, "c_abi_demo")
    cmd = [_hipcc(), "-O2", "-std=c++17", "--offload-arch=gfx950", "-Wno-unused-command-line-argument", "-Wno-unused-result",
           "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_demo.cpp"),
           "-L" + HERE, "-lsqa", "-Wl,-rpath," + HERE, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), r.stderr))
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    if "--demo" in sys.argv[1:]:
        build_demo()
    elif "--microbench" in sys.argv[1:]:
        build_microbench()
    else:
        build()
