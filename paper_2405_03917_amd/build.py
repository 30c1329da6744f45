"""Build libcq.so (gfx950) in-tree with hipcc.  Usable as ``python -m paper_2405_03917_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcq.so")
SOURCES = ["cq_api.hip", "cq_encode.hip", "cq_encode_mfma.hip", "cq_decode.hip", "cq_decode_rope.hip", "cq_chunk.hip", "cq_kmeans.hip", "cq_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results straight into VGPRs: the encode kernel consumes every accumulator value once
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wno-int-to-pointer-cast",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# per-file additions: the MFMA filter's running maxima must not be canonicalised (its header says why)
FILE_FLAGS = {"cq_encode_mfma.hip": ["-fno-honor-nans"]}


def build(verbose: bool = True) -> str:
    """Compile every source and link the shared library; always recompiles."""
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build()
    print(LIB)
    sys.exit(0)
