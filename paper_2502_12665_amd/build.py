"""Build the HIP library in-tree: paper_2502_12665_amd/liba2ats.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "liba2ats.so")
SOURCES = ["a2ats_api.hip", "build_lut.hip", "score_topk.hip", "sparse_attn.hip", "encode_keys.hip",
           "single_codebook.hip", "encode_single.hip", "codebook_fit.hip"]
HOST_SOURCES = ["attn_host.cpp"]   # host-only code (OpenMP + SIMD): the CPU side of the heterogeneous placement
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
         "-I", os.path.join(_ROOT, "include"), "-I", CSRC]
HOST_FLAGS = ["-x", "c++", "-O3", "-std=c++17", "-fPIC", "-fopenmp", "-Wall", "-I", os.path.join(_ROOT, "include")]


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source to an object in csrc/_build/ (in parallel) and link the library."""
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src in HOST_SOURCES:
        obj = os.path.join(bdir, src.replace(".cpp", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *HOST_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif out and verbose:
            print(f"[build] {src}:\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fopenmp", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
