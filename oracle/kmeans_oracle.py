"""ctypes front end of the CPU oracle for CQ's centroid learning (``kmeans_oracle.c``).

TEST INFRASTRUCTURE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module.  It builds the C
file with gcc on first use (``build()``), and it imports nothing from the GPU
package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kmeans_oracle.c")
_LIB = os.path.join(_HERE, "libkmeans_oracle.so")
_lib = None


def _has_fma() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            return " fma " in f.read().replace("\n", " ")
    except OSError:
        return False


def build(force: bool = False) -> str:
    """Compile kmeans_oracle.c -> libkmeans_oracle.so.  No contraction of a*b+c by the compiler:
    the fused multiply-adds of the distance are the explicit fmaf() calls only."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=gnu11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]
        if _has_fma():
            cmd.append("-mfma")         # fmaf() becomes the hardware instruction (same result, faster)
        subprocess.check_call(cmd + ["-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # CQ_KMEANS_ORACLE_LIB names a library built elsewhere (the host-sanitizer run of the tests), taken as it is
        override = os.environ.get("CQ_KMEANS_ORACLE_LIB")
        if not override:
            build()
        lib = ctypes.CDLL(override or _LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        i64, ci = ctypes.c_int64, ctypes.c_int
        lib.cq_oracle_kmeanspp.restype = ci
        lib.cq_oracle_kmeanspp.argtypes = [u16p, i64, f32p, i64, i64, ci, ci, u64p, i32p, f32p]
        lib.cq_oracle_lloyd.restype = ci
        lib.cq_oracle_lloyd.argtypes = [u16p, i64, f32p, i64, i64, ci, ci, ci, f32p, u16p, f64p]
        lib.cq_oracle_kmeans_objective.restype = ci
        lib.cq_oracle_kmeans_objective.argtypes = [u16p, i64, f32p, i64, i64, ci, ci, f32p, f64p, u16p]
        lib.cq_oracle_integer_weights.restype = ci
        lib.cq_oracle_integer_weights.argtypes = [f32p, i64, i64, u32p]
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctype))


def _x(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x)
    if x.dtype != np.float16 or x.ndim != 2:
        raise TypeError("x must be fp16 [n, D]")
    return x


def _w(w, n: int, G: int):
    if w is None:
        return None
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.shape != (n, G):
        raise ValueError(f"weights must be [n, G] = {(n, G)}, got {w.shape}")
    return w


def kmeanspp(x: np.ndarray, c: int, K: int, rnd: np.ndarray, w=None) -> Tuple[np.ndarray, np.ndarray]:
    """k-means++ for every group: x fp16 [n, D], rnd uint64 [G, K] -> (picks int32 [G, K],
    centres fp32 [G, K, c])."""
    x = _x(x)
    n, D = x.shape
    G = D // c
    rnd = np.ascontiguousarray(rnd, dtype=np.uint64)
    if rnd.shape != (G, K):
        raise ValueError("rnd must be [G, K]")
    w = _w(w, n, G)
    picks = np.empty((G, K), dtype=np.int32)
    cent = np.empty((G, K, c), dtype=np.float32)
    rc = _load().cq_oracle_kmeanspp(_ptr(x.view(np.uint16), ctypes.c_uint16), D, _ptr(w, ctypes.c_float), n, D, c, K,
                                    _ptr(rnd, ctypes.c_uint64), _ptr(picks, ctypes.c_int32), _ptr(cent, ctypes.c_float))
    if rc:
        raise ValueError(f"cq_oracle_kmeanspp failed ({rc})")
    return picks, cent


def lloyd(x: np.ndarray, c: int, cent: np.ndarray, n_iter: int, w=None):
    """n_iter Lloyd iterations from fp32 centroids [G, K, c] -> (centroids fp32, assignment uint16
    [G, n] of the last assignment step, objective fp64 [G, n_iter])."""
    x = _x(x)
    n, D = x.shape
    G = D // c
    cent = np.array(cent, dtype=np.float32, order="C", copy=True)
    K = cent.shape[1]
    if cent.shape != (G, K, c):
        raise ValueError("centroids must be [G, K, c]")
    w = _w(w, n, G)
    assign = np.zeros((G, n), dtype=np.uint16)
    obj = np.zeros((G, max(n_iter, 1)), dtype=np.float64)
    rc = _load().cq_oracle_lloyd(_ptr(x.view(np.uint16), ctypes.c_uint16), D, _ptr(w, ctypes.c_float), n, D, c, K,
                                 n_iter, _ptr(cent, ctypes.c_float), _ptr(assign, ctypes.c_uint16),
                                 _ptr(obj, ctypes.c_double))
    if rc:
        raise ValueError(f"cq_oracle_lloyd failed ({rc})")
    return cent, assign, obj[:, :n_iter]


def objective(x: np.ndarray, c: int, cent: np.ndarray, w=None):
    """Weighted objective per group of fp32 centroids [G, K, c] -> (fp64 [G], assignment [G, n])."""
    x = _x(x)
    n, D = x.shape
    G = D // c
    cent = np.ascontiguousarray(cent, dtype=np.float32)
    K = cent.shape[1]
    w = _w(w, n, G)
    obj = np.zeros(G, dtype=np.float64)
    assign = np.zeros((G, n), dtype=np.uint16)
    rc = _load().cq_oracle_kmeans_objective(_ptr(x.view(np.uint16), ctypes.c_uint16), D, _ptr(w, ctypes.c_float), n, D,
                                            c, K, _ptr(cent, ctypes.c_float), _ptr(obj, ctypes.c_double),
                                            _ptr(assign, ctypes.c_uint16))
    if rc:
        raise ValueError(f"cq_oracle_kmeans_objective failed ({rc})")
    return obj, assign


def integer_weights(w, n: int, G: int) -> np.ndarray:
    """The integer weights [G, n] the learning uses for fp32 weights [n, G] (None: all ones)."""
    w = _w(w, n, G)
    wq = np.zeros((G, n), dtype=np.uint32)
    rc = _load().cq_oracle_integer_weights(_ptr(w, ctypes.c_float), n, G, _ptr(wq, ctypes.c_uint32))
    if rc:
        raise ValueError("cq_oracle_integer_weights failed")
    return wq


def fit(x: np.ndarray, c: int, K: int, rnd: np.ndarray, n_iter: int, w=None):
    """k-means++ then n_iter Lloyd iterations -> (centroids fp16 [G, K, c] (the fp32 result rounded
    to nearest even), centroids fp32, assignment of the last assignment step, objective [G, n_iter])."""
    _, c0 = kmeanspp(x, c, K, rnd, w)
    cent, assign, obj = lloyd(x, c, c0, n_iter, w)
    return cent.astype(np.float16), cent, assign, obj
