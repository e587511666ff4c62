"""Builds libvidiq.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc.

Usage: python -m paper_2406_02540_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libvidiq.so")
CEILINGS_PATH = os.path.join(PKG_DIR, "vq_ceilings")  # stand-alone program, see csrc/vq_ceilings.hip
SOURCES = ["vq_api.hip", "vq_quantize.hip", "vq_fused.hip", "vq_fused_gelu.hip", "vq_gemm.hip", "vq_gemm_192.hip", "vq_gemm_small.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-ffp-contract=off",          # every fp32 operation rounds on its own
    "-fno-fast-math",
    # packed-fp32 instructions are not used in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = True) -> str:
    """Compiles every source for gfx950 and links the shared library. Always recompiles."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    for src, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"hipcc failed on {src}")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB_PATH)
    # the ceilings probe (register-only MFMA loop, copy kernel): its own small executable
    tmp = CEILINGS_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *[f for f in HIPCC_FLAGS if f != "-fPIC"], os.path.join(CSRC, "vq_ceilings.hip"), "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, CEILINGS_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build()
    print("built", LIB_PATH)
    sys.exit(0)
