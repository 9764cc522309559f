"""Build step of the HIP library: one hipcc call over csrc/*.hip for gfx950, output in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libmoe_mi355x.so")


def sources():
    return sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))


def build_library(verbose: bool = False) -> str:
    """Compile every kernel and the C ABI into libmoe_mi355x.so (cross-compiles without a GPU)."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc"),
           # keep hipcc from forming packed-fp32 instructions out of ordinary float code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + os.environ.get("MOE_EXTRA_HIPCC_FLAGS", "").split() + sources()
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose:
        print(out)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(verbose="-v" in sys.argv))
