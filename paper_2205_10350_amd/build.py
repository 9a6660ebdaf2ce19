"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libad_mi355x.so")
SOURCES = ["ad_hostlogic.cpp", "ad_api.cpp", "ad_kernels.hip", "ad_attention_long.hip"]
# -amdgpu-mfma-vgpr-form: MFMA results go to ordinary vector registers, not to the accumulation
# registers and back through copies before every vector instruction that reads them (masks, maxima,
# epilogues): 1-2 % of the forward, no spills.
# -amdgpu-kernarg-preload-count=16: the first 64 bytes of a kernel's arguments are in scalar registers
# when a wave starts instead of being loaded (in two or three dependent steps) by its first
# instructions; the kernels order their arguments for it: 4-6 % of the forward.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form=1", "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 target feature and says so: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compiles every source (one hipcc process each, side by side) and links the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    jobs = []
    for s in SOURCES:
        o = os.path.join(objdir, os.path.splitext(s)[0] + ".o")
        objs.append(o)
        jobs.append([hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-c", os.path.join(HERE, "csrc", s), "-o", o])
    with ThreadPoolExecutor(max_workers=len(jobs)) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
