"""ctypes front end of the fp64 CPU oracle (``cq_oracle.c``).

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
_SRC = os.path.join(_HERE, "cq_oracle.c")
_LIB = os.path.join(_HERE, "libcq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile cq_oracle.c -> libcq_oracle.so (gcc, -O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # CQ_ORACLE_LIB names a library built elsewhere (the host-sanitizer run of the tests), taken as it is
        override = os.environ.get("CQ_ORACLE_LIB")
        if not override:
            build()
        lib = ctypes.CDLL(override or _LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.cq_oracle_half_to_double.restype = ctypes.c_double
        lib.cq_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.cq_oracle_max_threads.restype = ctypes.c_int
        lib.cq_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.cq_oracle_encode.restype = ctypes.c_int
        lib.cq_oracle_encode.argtypes = [u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         u16p, ctypes.c_int, ctypes.c_int, u16p, f64p, f64p]
        lib.cq_oracle_dequantize.restype = ctypes.c_int
        lib.cq_oracle_dequantize.argtypes = [u16p, ctypes.c_int64, ctypes.c_int64, u16p,
                                             ctypes.c_int, ctypes.c_int, f64p]
        lib.cq_oracle_attention.restype = ctypes.c_int
        lib.cq_oracle_attention.argtypes = [u16p, u16p, u16p, u16p, u16p, ctypes.c_double,
                                            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_int64, ctypes.c_int, ctypes.c_int, i32p,
                                            f64p, f64p, f64p]
        lib.cq_oracle_attention_rope.restype = ctypes.c_int
        lib.cq_oracle_attention_rope.argtypes = [u16p, u16p, u16p, u16p, u16p, ctypes.c_double,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_int64, ctypes.c_int, ctypes.c_int, i32p,
                                                 ctypes.c_double, ctypes.c_int64, f64p, f64p, f64p]
        _lib = lib
    return _lib


def _u16(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _f64(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _bits(a: np.ndarray) -> np.ndarray:
    """fp16 array -> contiguous uint16 view of its bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("expected float16, got %s" % a.dtype)
    return a.view(np.uint16)


def max_threads() -> int:
    return int(_load().cq_oracle_max_threads())


def set_threads(n: int) -> None:
    _load().cq_oracle_set_threads(int(n))


def half_to_double(bits: int) -> float:
    return float(_load().cq_oracle_half_to_double(int(bits)))


def encode(x: np.ndarray, centroids: np.ndarray, with_distances: bool = False):
    """x fp16 [T, D], centroids fp16 [G, 2^b, c] -> codes uint16 [T, G]
    (and, if asked, the best and second-best squared distances, fp64 [T, G])."""
    lib = _load()
    xb = _bits(x)
    cb = _bits(centroids)
    T, D = xb.shape
    G, K, c = cb.shape
    b = int(K).bit_length() - 1
    if (1 << b) != K or G * c != D:
        raise ValueError("codebook shape does not match x")
    codes = np.empty((T, G), dtype=np.uint16)
    best = np.empty((T, G), dtype=np.float64) if with_distances else None
    second = np.empty((T, G), dtype=np.float64) if with_distances else None
    rc = lib.cq_oracle_encode(_u16(xb), T, D, D, _u16(cb), c, b, _u16(codes), _f64(best), _f64(second))
    if rc != 0:
        raise ValueError("cq_oracle_encode rejected its arguments")
    if with_distances:
        return codes, best, second
    return codes


def dequantize(codes: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """codes uint16 [T, G], centroids fp16 [G, 2^b, c] -> fp64 [T, G*c]."""
    lib = _load()
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    cb = _bits(centroids)
    T, G = codes.shape
    G2, K, c = cb.shape
    b = int(K).bit_length() - 1
    if G2 != G:
        raise ValueError("codebook shape does not match codes")
    out = np.empty((T, G * c), dtype=np.float64)
    rc = lib.cq_oracle_dequantize(_u16(codes), T, G * c, _u16(cb), c, b, _f64(out))
    if rc != 0:
        raise ValueError("cq_oracle_dequantize rejected its arguments")
    return out


def attention(q: np.ndarray, k_codes: np.ndarray, v_codes: np.ndarray,
              k_centroids: np.ndarray, v_centroids: np.ndarray, scale: float,
              n_kv_heads: int, seq_lens: Optional[np.ndarray] = None,
              want_scores: bool = False, want_probs: bool = False,
              rope_base: Optional[float] = None, pos_offset: int = 0):
    """q fp16 [B, Hq, d]; codes uint16 [B, T, G]; centroids fp16 [G, 2^b, c].
    Returns out fp64 [B, Hq, d] (plus scores / probabilities [B, Hq, T] if asked).
    With rope_base the cached keys are pre-rotation keys: the key of cached token t is rotated
    to position t + pos_offset (pairs (i, i + d/2), angle position * rope_base^(-2i/d)) before
    the dot product with q, which is taken as already rotated."""
    lib = _load()
    qb = _bits(q)
    kc = np.ascontiguousarray(k_codes, dtype=np.uint16)
    vc = np.ascontiguousarray(v_codes, dtype=np.uint16)
    ckb = _bits(k_centroids)
    cvb = _bits(v_centroids)
    B, Hq, d = qb.shape
    B2, T, G = kc.shape
    G2, K, c = ckb.shape
    b = int(K).bit_length() - 1
    if B2 != B or vc.shape != kc.shape or cvb.shape != ckb.shape or G2 != G or G * c != n_kv_heads * d:
        raise ValueError("inconsistent shapes")
    out = np.empty((B, Hq, d), dtype=np.float64)
    scores = np.full((B, Hq, T), np.nan) if want_scores else None
    probs = np.zeros((B, Hq, T)) if want_probs else None
    sl = None
    slp = ctypes.POINTER(ctypes.c_int32)()
    if seq_lens is not None:
        sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
        if sl.shape != (B,):
            raise ValueError("seq_lens must have shape [B]")
        slp = sl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    if rope_base is None:
        rc = lib.cq_oracle_attention(_u16(qb), _u16(kc), _u16(vc), _u16(ckb), _u16(cvb), float(scale),
                                     B, Hq, n_kv_heads, d, T, c, b, slp, _f64(out), _f64(scores), _f64(probs))
    else:
        rc = lib.cq_oracle_attention_rope(_u16(qb), _u16(kc), _u16(vc), _u16(ckb), _u16(cvb), float(scale),
                                          B, Hq, n_kv_heads, d, T, c, b, slp, float(rope_base), int(pos_offset),
                                          _f64(out), _f64(scores), _f64(probs))
    if rc != 0:
        raise ValueError("cq_oracle_attention failed (rc=%d)" % rc)
    res: Tuple = (out,)
    if want_scores:
        res += (scores,)
    if want_probs:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def chunk_attention(q: np.ndarray, k_codes: np.ndarray, v_codes: np.ndarray,
                    k_centroids: np.ndarray, v_centroids: np.ndarray, scale: float,
                    n_kv_heads: int, seq_lens: Optional[np.ndarray] = None,
                    rope_base: Optional[float] = None) -> np.ndarray:
    """Causal attention of the LAST m tokens of each sequence over its coded cache: Eq. 1 of the
    paper applied once per query token, each over the cached tokens up to and including its own
    position (the cache already holds the codes of the m tokens).  With `rope_base` the cached keys
    are pre-rotation keys (Section 3.2) and attention() rotates each to its position; the query
    tokens arrive rotated.

    q fp16 [B, m, Hq, d]: query j of sequence n sits at position t_n - m + j, where t_n =
    seq_lens[n] (default: all T cached tokens), and attends to tokens 0 .. t_n - m + j.
    Returns fp64 [B, m, Hq, d].  One call of attention() per query token: no blocking, no reuse."""
    q = np.asarray(q)
    B, m, Hq, d = q.shape
    T = k_codes.shape[1]
    t_n = np.full(B, T, dtype=np.int64) if seq_lens is None else np.asarray(seq_lens, dtype=np.int64)
    if np.any(t_n < m) or np.any(t_n > T):
        raise ValueError("every sequence must hold its m query tokens: m <= seq_len <= T")
    out = np.empty((B, m, Hq, d), dtype=np.float64)
    for j in range(m):
        lens = (t_n - m + j + 1).astype(np.int32)
        out[:, j] = attention(np.ascontiguousarray(q[:, j]), k_codes, v_codes, k_centroids, v_centroids, scale,
                              n_kv_heads, seq_lens=lens, rope_base=rope_base)
    return out
