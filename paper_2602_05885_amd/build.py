"""Builds the HIP library in-tree: python -m paper_2602_05885_amd.build"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpg_head.so")
SOURCES = ["api.hip", "kernels_gemm.hip", "kernels_rows.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def hipcc() -> str:
    for c in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True) -> str:
    """Compiles every source for gfx950 and links libpg_head.so next to this file."""
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}\n{out}")
        objs.append(obj)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    # stand-alone measurement tools (their failure must not fail the product build): the tile engine's main
    # loop alone, the persistent form of the forward kernel next to the one-workgroup-per-tile form, and the
    # in-kernel timeline of a vocab chunk's three launches
    for tool in ("tile_bench", "stream_bench", "tail_bench"):
        cmd = [cc, *[f for f in FLAGS if f != "-fPIC"], os.path.join(CSRC, tool + ".hip"), "-o", os.path.join(PKG, tool)]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        if r.returncode != 0 and verbose:
            print(f"warning: {tool} did not build (the library is unaffected)", flush=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
