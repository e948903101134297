"""Builds the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import concurrent.futures
import json
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libpipeoffload.so")
RESOURCES = os.path.join(PKG, "kernel_resources.json")  # per kernel: registers, scratch bytes per lane, occupancy
SOURCES = ["elementwise.hip", "gemm_generic.hip", "gemm_mfma.hip", "attention_generic.hip", "attention_mfma.hip",
           "schedule.cpp", "stage.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-sometimes-uninitialized", "-Wno-unknown-attributes",
         "-Rpass-analysis=kernel-resource-usage"]
_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"LDS Size \[bytes/block\]): (\S+)")


def _compile(src: str):
    """Compiles one source; returns (object path, {kernel: resource usage}) from the compiler's own report."""
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    usage, current, rest, skip = {}, None, [], 0
    for line in r.stderr.splitlines():
        if noise in line:
            continue
        if "[-Rpass-analysis=kernel-resource-usage]" in line:
            m = _REMARK.search(line)
            if m:
                key, val = m.group(1), m.group(2)
                if key == "Function Name":
                    current = usage.setdefault(val, {})
                elif current is not None:
                    current[key.split(" [")[0]] = int(val) if val.isdigit() else val
            skip = 2  # the two source-echo lines that follow every remark
            continue
        if skip:
            skip -= 1
            continue
        rest.append(line)
    err = "\n".join(rest)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj, usage


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    usage = {}
    for _, u in results:
        usage.update(u)
    with open(RESOURCES, "w") as f:
        json.dump(usage, f, indent=1, sort_keys=True)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
