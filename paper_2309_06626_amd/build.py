"""Builds libsparse_conv.so (gfx950) in-tree with hipcc.  Run: python -m paper_2309_06626_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsparse_conv.so")
SOURCES = ["plan.hip", "igemm_bf16.hip", "igemm_f16.hip", "igemm_f32.hip", "bandpp.hip", "bandtap.hip", "bandrow.hip", "igemm_panel.hip", "igemm_buf.hip", "igemm_slab.hip", "igemm_streamk.hip", "igemm_rowseg.hip", "mask_gen.hip", "depthwise.hip", "backward.hip", "probes.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-value",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src: str, extra_flags=(), obj_dir: str = OBJ) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def build_library(jobs: int = 8, extra_flags=(), out: str = LIB, obj_dir: str = OBJ) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags, obj_dir), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", out, *objs,
           "-Wl,-rpath,/opt/rocm/lib", "-Wl,--no-undefined"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return out


if __name__ == "__main__":
    # python -m paper_2309_06626_amd.build [--define NAME=VALUE ...] [--out PATH]: a development build beside the
    # library (time-stamp or probe macros of the kernels), with its own object folder
    import argparse

    ap = argparse.ArgumentParser()
    ap.add_argument("--define", action="append", default=[])
    ap.add_argument("--out", default=LIB)
    a = ap.parse_args()
    out = os.path.abspath(a.out)
    build_library(extra_flags=tuple("-D" + d for d in a.define), out=out,
                  obj_dir=OBJ if out == LIB else out + ".objs")
    print(out)
