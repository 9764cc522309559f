"""Build step of the HIP library: hipcc over csrc/*.hip for gfx950, output in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
# the in-tree library; MOE_LIB names another build of the same sources (e.g. one made with other MOE_EXTRA_HIPCC_FLAGS)
LIB = os.environ.get("MOE_LIB") or os.path.join(PKG, "libmoe_mi355x.so")


def sources():
    return sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))


def build_library(verbose: bool = False) -> str:
    """Compile every kernel and the C ABI into libmoe_mi355x.so (cross-compiles without a GPU): one hipcc -c per source
    file, side by side, then one link."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(ROOT, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc"),
             # keep hipcc from forming packed-fp32 instructions out of ordinary float code
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + os.environ.get("MOE_EXTRA_HIPCC_FLAGS", "").split()
    if verbose:
        flags.append("-Rpass-analysis=kernel-resource-usage")

    def run(cmd):
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        return out

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        return obj, run(["hipcc", "-c"] + flags + ["-o", obj, src])

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        done = list(ex.map(compile_one, sources()))
    out = "\n".join(o for _, o in done)
    out += run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in done])
    if verbose:
        print(out)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(verbose="-v" in sys.argv))
