"""Compile the HIP library in-tree for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfairkv.so")
SOURCES = [os.path.join(CSRC, "fairkv_api.hip"), os.path.join(CSRC, "fairkv_plan.cpp"),
           os.path.join(CSRC, "fairkv_place.cpp")]
HEADERS = [os.path.join(ROOT, "include", "fairkv.h"), os.path.join(ROOT, "include", "fairkv_measure.h")] + [os.path.join(CSRC, h) for h in ("common.h", "decode_mfma.h", "decode_valu.h", "pack.h", "stream_probe.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # MFMA accumulators in ordinary vector registers: the softmax rescales them with vector
           # instructions, and the accumulation-register form costs a copy in and out per tile
           "-mllvm", "-amdgpu-mfma-vgpr-form=1",
           "-Wall", "-Wextra", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
           "-I", os.path.join(ROOT, "include"), "-x", "hip", *SOURCES, "-o", LIB]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err:
        print(err)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force=True, verbose="-v" in sys.argv))
