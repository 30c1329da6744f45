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
    """Compile every source and link the shared library; always recompiles.  Objects go to a
    directory of this process's own (two builds at once cannot link each other's half-written
    objects); the finished library is moved into place in one step."""
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    objdir = tempfile.mkdtemp(prefix="libcq_build_")
    try:
        def compile_one(src):
            obj = os.path.join(objdir, src.replace(".hip", ".o"))
            cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj
        with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = LIB + f".tmp{os.getpid()}"
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    build()
    print(LIB)
    sys.exit(0)
