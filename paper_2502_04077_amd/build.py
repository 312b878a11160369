"""Builds libattnpred.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libattnpred.so")


def build_library(verbose: bool = False) -> str:
    srcs = sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))
    cmd = [
        "hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG_DIR, "csrc"),
        # keep the compiler from forming packed-fp32 VALU ops
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        # MFMA accumulators in ordinary VGPRs: no AGPR <-> VGPR copies around every chain
        "-mllvm", "-amdgpu-mfma-vgpr-form=1",
        *srcs, "-o", LIB_PATH,
    ]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        noise = "is not a recognized feature for this target"      # hipcc's host pass, harmless
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if noise not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libattnpred.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
