"""Builds libtangram.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import json
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtangram.so")
RESOURCES = os.path.join(HERE, "kernel_resources.json")   # written by every build, next to the library
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into one shared library; returns its path."""
    srcs = sources()
    deps = srcs + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [
        os.path.join(ROOT, "include", "tg.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB] + srcs
    cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    if verbose:
        print(" ".join(cmd))
    done = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    kernels = _resource_remarks(done.stderr)
    if done.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in done.stderr.splitlines() if "remark:" not in l)[-4000:])
    with open(RESOURCES, "w") as f:
        json.dump(kernels, f, indent=1, sort_keys=True)
    return LIB


def _resource_remarks(stderr: str) -> dict:
    """Registers, scratch and occupancy of every kernel, from the compiler's resource-usage remarks."""
    kernels, cur = {}, None
    for line in stderr.splitlines():
        m = re.search(r"remark:\s+(Function Name|VGPRs|AGPRs|TotalSGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                      r"LDS Size \[bytes/block\]):\s+(\S+)", line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = kernels.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return kernels


if __name__ == "__main__":
    print(build_library(verbose=True))
