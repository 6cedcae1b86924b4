"""Builds libtwgemm.so (HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libtwgemm.so")
SOURCES = ["api.cpp", "pack.cpp", "gemm_kernels.hip", "gemm_dma.hip", "gemm_tvw.hip", "gemm_i8.hip", "gemm_tvw_i8.hip", "prune.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instruction selection is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = False) -> str:
    srcs = [os.path.join(PKG, "csrc", s) for s in SOURCES]
    cmd = [HIPCC, *FLAGS, "-I" + os.path.join(ROOT, "include"), *srcs, "-o", LIB + ".tmp"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
    os.replace(LIB + ".tmp", LIB)
    if verbose:
        print(r.stderr)
    return LIB


def ensure_built() -> str:
    """Builds the library only if there is none (tests, the smoke check and the benchmark call
    this; the binding itself never builds and fails loudly when the library is missing)."""
    return LIB if os.path.exists(os.environ.get("TWGEMM_LIB") or LIB) else build()


if __name__ == "__main__":
    print(build(verbose=True))
