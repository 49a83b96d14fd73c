"""Compile the HIP sources into libspecexit.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# SPECEXIT_LIB names another output file and SPECEXIT_DEFS extra -D flags: side-by-side builds of kernel variants
LIB = os.environ.get("SPECEXIT_LIB") or os.path.join(HERE, "libspecexit.so")
SOURCES = ["api.hip", "gemm.hip", "gemm_wide.hip", "gemv.hip", "attn.hip", "attn_mfma.hip", "draft.hip", "accept_exit.hip", "kv_compact.hip", "tree.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = (["-Rpass-analysis=kernel-resource-usage"] if os.environ.get("SPECEXIT_RESOURCE_REMARKS") else []) + ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         # packed fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + os.environ.get("SPECEXIT_DEFS", "").split()


def build(verbose: bool = True) -> str:
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build") if not os.environ.get("SPECEXIT_LIB") else LIB + ".build"
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out)
        if p.returncode:
            failed = True
            print(f"compile of {src} failed", file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
