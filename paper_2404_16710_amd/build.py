"""Builds libls.so (the C-ABI library) in-tree with hipcc for gfx950.

Each translation unit is compiled to an object file (in parallel; the four decode-kernel
variants take most of the time), then linked into paper_2404_16710_amd/libls.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libls.so")
SOURCES = [
    "ls_kernels_bf16_hd128.hip", "ls_kernels_bf16_hd64.hip", "ls_kernels_f32_hd128.hip", "ls_kernels_f32_hd64.hip",
    "ls_launch.hip", "ls_prefill.hip", "ls_api.cpp",
]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # Inter-procedural register allocation: the few real (non-inlined) device functions are static,
    # so with it they no longer save and restore ~190 callee-saved registers per call (184 KB of
    # scratch traffic per workgroup each way, about 10 us per pass); a call that carries the "tail"
    # marker is excluded from that, hence no sibling-call marking.
    "-mllvm", "-enable-ipra", "-fno-optimize-sibling-calls",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)


def build(verbose: bool = True, jobs: int = 7) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    objs = [os.path.join(OBJDIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    cmds = [[HIPCC] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda c: _run(c, verbose), cmds))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
