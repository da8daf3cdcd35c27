"""Builds libstarattn.so (the C-ABI HIP library) and libstarcalib.so (the
benchmark's calibration kernels) in-tree with hipcc for gfx950.

Usage:  python -m paper_2411_17116_amd.build
The library is written next to this file so that it travels with the source
tree; nothing is installed outside the repository.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libstarattn.so")
SOURCES = ["api.hip", "kv_cache.hip", "rope.hip", "flash_f32.hip", "flash_bf16.hip",
           "decode_bf16.hip", "merge.hip"]
# the benchmark's calibration kernels: a library of their own, so that the
# product library holds nothing but the path
CALIB_LIB = os.path.join(HERE, "libstarcalib.so")
CALIB_SOURCES = ["calib.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = True, jobs: int = 6) -> str:
    """Compile every source for gfx950 and link the shared library."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES + CALIB_SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        if src in SOURCES:
            objs.append(obj)
        cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            for _, p in procs:
                if p.poll() is None:
                    p.wait()
                    break
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(ln for ln in out.splitlines()
                        if "packed-fp32-ops" not in ln)   # host pass does not know the feature
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    calib_objs = [os.path.join(objdir, src.replace(".hip", ".o")) for src in CALIB_SOURCES]
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *calib_objs, "-o", CALIB_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
