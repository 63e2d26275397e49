"""Build libsvdq.so in-tree with hipcc for gfx950 (no JIT cache: the .so must travel with the tree)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsvdq.so")

SOURCES = ["prepare.cpp", "act_kernel.hip", "gemm_w4a4_kernel.hip", "gemm_fp4_kernel.hip", "w8a8_kernels.hip", "w4a16_kernel.hip", "peak_probe.hip", "api.hip"]

# -packed-fp32-ops is switched OFF for all device code; no fast-math, no fp contraction:
# the quantizer's roundings must be exactly the IEEE single operations that are written.
COMMON = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fno-fast-math",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


# GEMM kernels only: MFMA results go to ordinary VGPRs.  The rescale consumes them on the vector ALU right away, and an
# AGPR destination would cost one v_accvgpr_read per partial sum.
MFMA_VGPR = {"gemm_w4a4_kernel.hip", "gemm_fp4_kernel.hip", "w8a8_kernels.hip", "peak_probe.hip"}


def build_library(verbose: bool = True, extra: list[str] | None = None) -> str:
    cc = hipcc()
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.rsplit(".", 1)[0] + ".o")
        cmd = [cc] + COMMON + (["-mllvm", "-amdgpu-mfma-vgpr-form"] if src in MFMA_VGPR else []) + (extra or [])
        if src.endswith(".cpp"):
            cmd += ["-x", "hip"]
        cmd += ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    cmd = [cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
