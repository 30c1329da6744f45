#!/usr/bin/env python3
"""Host-side sanitizer pass (CPU only; no GPU is touched and no device code is instrumented).

    python tests/host_sanitizers.py

1. Builds oracle/cq_oracle.c and oracle/kmeans_oracle.c with gcc -fsanitize=address,undefined and
   runs every `-m "not gpu"` test against those builds (AddressSanitizer's runtime preloaded into
   the interpreter; leak checking off, the interpreter itself never frees everything).
2. Builds libcq.so with the HOST code of every source instrumented (hipcc -Xarch_host
   -fsanitize=address -Xarch_host -fsanitize=undefined; the device code is compiled as usual)
   and runs tests/test_libcq_host.py -- every argument-validation path of the C ABI -- against
   it, with the compiler's own AddressSanitizer runtime preloaded.

Exit status 0 when both passes are clean.  Build products go to a temporary directory.
"""
import glob
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def run(cmd, env=None):
    print("+", " ".join(cmd), flush=True)
    return subprocess.call(cmd, cwd=ROOT, env=env)


def gcc_runtime(name):
    return subprocess.check_output(["gcc", f"-print-file-name={name}"], text=True).strip()


def main():
    tmp = tempfile.mkdtemp(prefix="cq_san_")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    # ---- pass 1: the oracle
    lib_o, lib_k = os.path.join(tmp, "libcq_oracle.so"), os.path.join(tmp, "libkmeans_oracle.so")
    if run(["gcc", *san, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib_o,
            os.path.join(ROOT, "oracle", "cq_oracle.c"), "-lm"]):
        return 1
    if run(["gcc", *san, "-std=gnu11", "-ffp-contract=off", "-mfma", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib_k,
            os.path.join(ROOT, "oracle", "kmeans_oracle.c"), "-lm"]):
        return 1
    env = dict(os.environ, CQ_ORACLE_LIB=lib_o, CQ_KMEANS_ORACLE_LIB=lib_k,
               LD_PRELOAD=":".join(x for x in (os.environ.get("LD_PRELOAD"), gcc_runtime("libasan.so")) if x),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    rc1 = run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"], env)
    # ---- pass 2: the library's host code
    from paper_2405_03917_amd import build as B
    objs = []
    hflags = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    for src in B.SOURCES:
        obj = os.path.join(tmp, src.replace(".hip", ".o"))
        flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1", "-g"]
        if run([B.HIPCC, *flags, *B.FILE_FLAGS.get(src, []), *hflags, "-c", os.path.join(B.CSRC, src), "-o", obj]):
            return 1
        objs.append(obj)
    lib = os.path.join(tmp, "libcq.so")
    if run([B.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan",
            "-o", lib, *objs]):
        return 1
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    env = dict(os.environ, LIBCQ_PATH=lib,
               LD_PRELOAD=":".join(x for x in (os.environ.get("LD_PRELOAD"), rt[0] if rt else None) if x),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    rc2 = run([sys.executable, "-m", "pytest", "tests/test_libcq_host.py", "-x", "-q", "-p", "no:cacheprovider"], env)
    print(f"oracle pass: {'clean' if rc1 == 0 else 'FAILED'}; library host-code pass: {'clean' if rc2 == 0 else 'FAILED'}")
    return 1 if (rc1 or rc2) else 0


if __name__ == "__main__":
    sys.exit(main())
