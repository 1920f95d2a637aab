"""Compile the HIP planner for gfx950 into paper_2309_08125_amd/lib/liboob_plan.so."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC_DIR = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "liboob_plan.so")


def sources():
    return sorted(glob.glob(os.path.join(SRC_DIR, "*.hip")))


def build(verbose: bool = False) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-fno-honor-nans", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", SRC_DIR, "-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    if verbose and err.strip():
        print(err)
    return LIB


def ensure_built() -> str:
    """Builds only if no library is there (tests, smoke and bench call this; a changed source
    needs an explicit build)."""
    return LIB if os.path.exists(LIB) else build()


if __name__ == "__main__":
    print(build(verbose=True))
