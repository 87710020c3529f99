"""Builds libegt.so (HIP kernels + C ABI) in-tree with hipcc for gfx950.

Every source is compiled to an object of its own (in parallel) and the objects are linked
into the shared library.  EGT_EXTRA_HIPCC_FLAGS adds flags for a developer build, e.g.
`-DEGT_TUNE` (launch-shape knobs read from the environment, see csrc/egt_tune.h) or
`-DEGT_ABLATE=<n>` (stages of the headline kernel switched off for timing, see
csrc/egt_mfma_m1.hip).  `python -m paper_2605_11582_amd.build --resource-usage` prints the
compiler's per-kernel register, LDS and scratch figures.
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libegt.so")
OBJ_DIR = os.path.join(PKG, "_build")
EXTRA_FLAGS = os.environ.get("EGT_EXTRA_HIPCC_FLAGS", "").split()


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _flags(csrc: str) -> list:
    # -ffp-contract=off: a multiply is fused with an add only where the source says fmaf, so
    # the same expression gives the same bits in every kernel that contains it
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-pthread", *EXTRA_FLAGS,
            "-I" + os.path.join(ROOT, "include"), "-I" + csrc]


def build(verbose: bool = False, resource_usage: bool = False, out: str = LIB) -> str:
    csrc = os.path.join(PKG, "csrc")
    srcs = sorted(glob.glob(os.path.join(csrc, "*.cpp")) + glob.glob(os.path.join(csrc, "*.hip")))
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = hipcc_path()
    extra = ["-Rpass-analysis=kernel-resource-usage"] if resource_usage else []

    def compile_one(src: str):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        cmd = [hipcc, *_flags(csrc), *extra, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        return src, obj, res

    jobs = min(len(srcs), int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 4, 16)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_one, srcs))
    for src, _, res in results:
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {os.path.basename(src)}:\n" + res.stdout + res.stderr)
        if resource_usage:
            sys.stdout.write(res.stderr)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", *[o for _, o, _ in results],
            "-o", out + ".tmp"]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    os.replace(out + ".tmp", out)
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, resource_usage="--resource-usage" in sys.argv))
