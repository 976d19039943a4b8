"""Build libdip.so for gfx950 with hipcc, in-tree (paper_2412_01380_amd/lib/libdip.so)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIBPATH = os.path.join(LIBDIR, "libdip.so")
SOURCES = ["dip_api.hip", "dip_select.hip", "dip_gemv.hip", "dip_batched.hip", "dip_tier.hip"]
# dip_fused.hip is compiled once per (segments, weight type): six objects built in parallel
FUSED_VARIANTS = [(nseg, dtype) for nseg in (1, 2) for dtype in (0, 1, 2)]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                       # scores need separate multiply and divide
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(LIBDIR, exist_ok=True)
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in FLAGS if f]
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for nseg, dtype in FUSED_VARIANTS:
        obj = os.path.join(objdir, f"dip_fused_{nseg}_{dtype}.o")
        objs.append(obj)
        cmd = [hipcc, *flags, f"-DDIP_FUSED_NSEG={nseg}", f"-DDIP_FUSED_DTYPE={dtype}",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, "dip_fused.hip"), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((f"dip_fused.hip[{nseg},{dtype}]",
                      subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIBPATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIBPATH


if __name__ == "__main__":
    build()
    print("built", LIBPATH)
