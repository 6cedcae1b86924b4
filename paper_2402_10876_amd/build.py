"""Builds libtwgemm.so (HIP for gfx950) in-tree with hipcc.

A digest of the sources, headers and compiler flags is written next to the library
(`libtwgemm.so.srchash`); `ensure_built()` rebuilds when that digest no longer matches the
tree, so that a test run, the smoke check or the benchmark can never measure a library that
is older than the sources beside it."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libtwgemm.so")
HASH_FILE = LIB + ".srchash"
SOURCES = ["api.cpp", "pack.cpp", "gemm_kernels.hip", "gemm_dma.hip", "gemm_tvw.hip", "gemm_i8.hip", "gemm_tvw_i8.hip", "prune.hip", "pack_dev.hip", "calibrate.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instruction selection is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def source_hash() -> str:
    """Digest of everything the library is built from: csrc/*, include/*.h and the flags."""
    h = hashlib.sha256(" ".join(FLAGS + SOURCES).encode())
    files = sorted(glob.glob(os.path.join(PKG, "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for p in files:
        if os.path.isfile(p):
            h.update(os.path.basename(p).encode() + b"\0")
            with open(p, "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def built_hash() -> str | None:
    """Digest recorded when the library in the tree was built (None: no library, or no record)."""
    if not (os.path.exists(LIB) and os.path.exists(HASH_FILE)):
        return None
    with open(HASH_FILE) as f:
        return f.read().strip()


def build(verbose: bool = False) -> str:
    srcs = [os.path.join(PKG, "csrc", s) for s in SOURCES]
    digest = source_hash()
    cmd = [HIPCC, *FLAGS, "-I" + os.path.join(ROOT, "include"), *srcs, "-o", LIB + ".tmp"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
    os.replace(LIB + ".tmp", LIB)
    with open(HASH_FILE, "w") as f:
        f.write(digest + "\n")
    if verbose:
        print(r.stderr)
    return LIB


def ensure_built() -> str:
    """Loads what is built when it matches the sources, builds otherwise (tests, the smoke check
    and the benchmark call this; the binding itself never builds and fails loudly when the
    library is missing).  A library named by TWGEMM_LIB is the caller's responsibility."""
    if os.environ.get("TWGEMM_LIB"):
        return os.environ["TWGEMM_LIB"]
    if built_hash() == source_hash():
        return LIB
    return build()


def describe() -> str:
    """Which binary is in use: path and the digest of the sources it was built from."""
    if os.environ.get("TWGEMM_LIB"):
        return f"{os.environ['TWGEMM_LIB']} (TWGEMM_LIB, digest unknown)"
    return f"{LIB} (sources {built_hash()})"


if __name__ == "__main__":
    print(build(verbose=True))
