"""Build-time check of the kernels' split asynchronous loads.

The kernels issue LDS reads (ds_read_*) and scalar loads (s_load_*) from inline
assembly and wait for them in a LATER inline-assembly statement
(`s_waitcnt lgkmcnt(0)`), so that matrix instructions and copies can be issued in
between.  The compiler does not know that the destination registers of such a
load are not valid until the wait; it is free to copy or reuse them right after
the load statement (register coalescing of a loop-carried value does exactly
that).  This script compiles each kernel source to assembly and walks every
kernel in layout order (fall-through paths; the pending set is dropped at a label
that follows an unconditional jump): a register written by a load inside an
inline-assembly block is "pending" until the next `s_waitcnt` with `lgkmcnt(0)`;
any instruction that names a pending register before that wait is reported.

    python -m paper_2402_10876_amd.check_async_asm          # exit status 1 on a finding
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
KERNEL_SOURCES = ["gemm_kernels.hip", "gemm_dma.hip", "gemm_tvw.hip", "gemm_i8.hip", "gemm_tvw_i8.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "--cuda-device-only", "-S", "-Wno-unused-command-line-argument"]

_REG = re.compile(r"\b([vsa])(?:(\d+)|\[(\d+):(\d+)\])")
_ASYNC = re.compile(r"^(ds_read\w*|ds_load\w*|s_load_\w+|s_buffer_load_\w+)$")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(2) is not None:
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(1), i) for i in range(int(m.group(3)), int(m.group(4)) + 1))
    return out


def check_assembly(asm_text: str):
    """Returns a list of (kernel, line number, instruction, registers) findings."""
    findings = []
    kernel, in_app, pending, prev_op = None, False, {}, ""
    for ln, raw in enumerate(asm_text.split("\n"), 1):
        line = raw.strip()
        if line.startswith(";;#ASMSTART"):
            in_app = True
            continue
        if line.startswith(";;#ASMEND"):
            in_app = False
            continue
        code = line.split(";")[0].strip()
        if not code:
            continue
        if code.endswith(":"):
            if raw[0].isspace():
                continue
            if code.startswith("."):               # a local label: reached by fall-through unless the
                if prev_op in ("s_branch", "s_endpgm", "s_setpc_b64"):   # block before it ends in a jump
                    pending = {}
            else:
                kernel, pending = code[:-1], {}    # a new function
            continue
        if code.startswith("."):
            continue
        parts = code.split(None, 1)
        op, args = parts[0], (parts[1] if len(parts) > 1 else "")
        prev_op = op
        if op == "s_waitcnt":
            if "lgkmcnt(0)" in args:
                pending = {}
            continue
        if op == "s_endpgm":
            pending = {}
            continue
        if in_app and _ASYNC.match(op):
            dst_txt, _, src_txt = args.partition(",")
            bad = _regs(src_txt) & set(pending)
            if bad:
                findings.append((kernel, ln, code, sorted(bad)))
            for r in _regs(dst_txt):
                pending[r] = ln
            continue
        bad = _regs(args) & set(pending)
        if bad:
            findings.append((kernel, ln, code, sorted(bad)))
    return findings


def compile_to_asm(src: str) -> str:
    with tempfile.TemporaryDirectory() as td:
        out = os.path.join(td, "k.s")
        cmd = [HIPCC, *FLAGS, "-I" + os.path.join(ROOT, "include"), os.path.join(PKG, "csrc", src), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + " ".join(cmd) + "\n" + r.stderr[-3000:])
        return open(out).read()


def check_sources(sources=KERNEL_SOURCES):
    with ThreadPoolExecutor(max_workers=len(sources)) as ex:
        texts = list(ex.map(compile_to_asm, sources))
    res = []
    for src, text in zip(sources, texts):
        res += [(src,) + f for f in check_assembly(text)]
    return res


def main():
    res = check_sources()
    for src, kernel, ln, code, regs in res:
        print(f"{src}: {kernel}: line {ln}: `{code}` touches {regs} before the wait for its load")
    print(f"{len(res)} finding(s)")
    return 1 if res else 0


if __name__ == "__main__":
    sys.exit(main())
