"""Build the HIP library for gfx950 with hipcc, in-tree (``paper_2510_11958_amd/libdmtd.so``)."""
from __future__ import annotations

import os
import re
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libdmtd.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "dmtd.hip")]
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in SGPRs at wave launch instead of through a first dependent load
    # (the latency-bound attention kernels start ~0.2 us earlier; by-value argument structs are not covered)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    # per-kernel register and scratch figures on stderr: build_library() refuses a build whose matrix-core kernels spill
    "-Rpass-analysis=kernel-resource-usage",
]


def spilling_mfma_kernels(remarks: str) -> list:
    """Names of the *_mfma_kernel instantiations whose resource-usage remarks report a scratch size above zero."""
    bad, name = [], None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name and "_mfma_kernel" in name and int(m.group(1)) > 0:
            bad.append(f"{name} ({m.group(1)} bytes/lane)")
    return bad


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stderr)
    spilled = spilling_mfma_kernels(res.stderr)
    if spilled:
        # a weight-streaming kernel that spills to scratch still computes the right values, several times slower
        raise RuntimeError("matrix-core kernels use scratch memory (register spills): " + ", ".join(spilled))
    if verbose:
        print(" ".join(cmd))
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
