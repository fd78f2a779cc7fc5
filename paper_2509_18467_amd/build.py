"""Builds liblawcat.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "liblawcat.so")
SOURCES = ["api.hip", "conv1d.hip", "feature_map.hip", "gate_project.hip", "gla_backward.hip", "conv1d_backward.hip", "gla_recurrent.hip", "gla_chunk.hip", "gla_chunk_d64.hip", "gla_chunk_d128.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off on purpose: some of their forms have given wrong results on the test machines
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-sanitize", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, out: str | None = None) -> str:
    """Compile and link.  `out` (or the environment variable LAWCAT_LIB_OUT) names another output file, with its
    own object directory beside it, so that an experimental build never replaces the in-tree library that the
    tests and bench.py load."""
    out = out or os.environ.get("LAWCAT_LIB_OUT") or LIB
    objdir = os.path.join(_HERE, "_build") if out == LIB else out + ".objs"
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        extra = os.environ.get("LAWCAT_EXTRA_FLAGS", "").split()
        cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
