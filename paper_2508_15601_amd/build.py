"""Build libtm_w4.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libtm_w4.so")
SOURCES = ["tm_w4_api.hip", "tm_w4_pack.hip", "tm_w4_skinny.hip", "tm_w4_stream.hip", "tm_w4_stream_grouped.hip", "tm_w4_streamx.hip", "tm_w4_streamx64.hip", "tm_w4_skinny_w8.hip", "tm_w4_skinny_f8.hip", "tm_w4_tile_small.hip", "tm_w4_tile_large.hip", "tm_w4_tile32.hip",
           "tm_w4_tile_kgroup.hip", "tm_w4_tile_grouped.hip", "tm_w4_tile_w8.hip", "tm_attn.hip"]
# per-file extra flags (see the header comment of each file)
EXTRA = {"tm_w4_tile_small.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_kgroup.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_grouped.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_w8.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, jobs: int = 4) -> str:
    """Compile every translation unit and link the shared library.  Always rebuilds."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = LIB
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, *EXTRA.get(src, []), "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        noise = "is not a recognized feature for this target"
        out = "\n".join(l for l in out.splitlines() if noise not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if out.strip():
            print(out, file=sys.stderr)


if __name__ == "__main__":
    print(build(verbose=True))
