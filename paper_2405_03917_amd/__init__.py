"""Python binding of libcq, the MI355X-native hot path of Coupled Quantization (CQ).

Argument marshalling only: every function here forwards to the C-ABI entry point of the same
name in ``libcq.so`` (declared in ``include/libcq.h``); all arithmetic runs in the library's HIP
kernels.  PyTorch supplies device memory and streams.  There is no fallback: if the shared
library has not been built (``python -m paper_2405_03917_amd.build``) importing the functions
works but the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
# (LIBCQ_PATH names a build of the library elsewhere, e.g. the host-sanitizer build of the tests)
LIB_PATH = os.environ.get("LIBCQ_PATH") or os.path.join(_PKG, "libcq.so")

CQ_OK = 0
CQ_ERR_INVALID_ARG = 1
CQ_ERR_UNSUPPORTED = 2
CQ_ERR_WORKSPACE_TOO_SMALL = 3
CQ_ERR_HIP = 4
TILE_TOKENS = 64

EXPORTS = (
    "cq_version", "cq_status_string", "cq_format_check", "cq_code_bytes_per_token_head",
    "cq_cache_bytes", "cq_encode", "cq_encode_kv", "cq_decode_default_split", "cq_decode_workspace_bytes",
    "cq_decode_attention", "cq_decode_attention_static", "cq_decode_step", "cq_dequantize", "cq_paged_cache_bytes", "cq_encode_kv_paged",
    "cq_decode_attention_paged", "cq_decode_step_paged", "cq_kmeans_workspace_bytes", "cq_kmeans_fit",
    "cq_fused_format", "cq_expand_codebook", "cq_chunk_default_split", "cq_chunk_workspace_bytes", "cq_chunk_attention", "cq_chunk_attention_paged",
    "cq_layer_table_bytes", "cq_layer_table_fill", "cq_decode_step_layers",
    "cq_rope_table_bytes", "cq_rope_table", "cq_decode_rope_default_split", "cq_decode_attention_rope",
    "cq_decode_attention_rope_paged", "cq_decode_step_rope", "cq_decode_step_rope_paged",
    "cq_chunk_rope_workspace_bytes", "cq_chunk_attention_rope", "cq_chunk_attention_rope_paged",
    "cq_probe_stream_read", "cq_probe_copy", "cq_probe_mfma",
)


class CQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


class _Format(ctypes.Structure):
    _fields_ = [("c", ctypes.c_int32), ("b", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32)]


class _LayerIO(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("q", "x_k_new", "x_v_new", "k_codes", "v_codes", "k_centroids",
                                                "v_centroids", "out")]


class _PageTable(ctypes.Structure):
    _fields_ = [("n_pages", ctypes.c_int32), ("max_tiles", ctypes.c_int32), ("row_stride", ctypes.c_int64),
                ("block_table", ctypes.c_void_p)]


@dataclass(frozen=True)
class CQFormat:
    """CQ-<c>c<b>b (Section 3.2 of the paper) on ``n_kv_heads`` heads of ``head_dim`` channels."""
    c: int
    b: int
    head_dim: int
    n_kv_heads: int

    def _c(self) -> _Format:
        return _Format(self.c, self.b, self.head_dim, self.n_kv_heads)

    @property
    def channels(self) -> int:
        return self.head_dim * self.n_kv_heads

    @property
    def groups(self) -> int:
        return self.channels // self.c


_lib = None


def load() -> ctypes.CDLL:
    """dlopen libcq.so and declare its prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2405_03917_amd.build` "
            "(there is no non-HIP fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    fp = ctypes.POINTER(_Format)
    vp = ctypes.c_void_p
    i32 = ctypes.c_int32
    i64 = ctypes.c_int64
    lib.cq_version.restype = i32
    lib.cq_version.argtypes = []
    lib.cq_status_string.restype = ctypes.c_char_p
    lib.cq_status_string.argtypes = [ctypes.c_int]
    lib.cq_format_check.restype = ctypes.c_int
    lib.cq_format_check.argtypes = [fp]
    lib.cq_code_bytes_per_token_head.restype = ctypes.c_size_t
    lib.cq_code_bytes_per_token_head.argtypes = [fp]
    lib.cq_cache_bytes.restype = ctypes.c_size_t
    lib.cq_cache_bytes.argtypes = [fp, i32, i32]
    lib.cq_encode.restype = ctypes.c_int
    lib.cq_encode.argtypes = [vp, i64, i64, vp, fp, i32, i32, vp, i32, i32, vp]
    lib.cq_encode_kv.restype = ctypes.c_int
    lib.cq_encode_kv.argtypes = [vp, vp, i64, i64, vp, vp, fp, i32, i32, vp, vp, i32, i32, vp]
    lib.cq_decode_default_split.restype = i32
    lib.cq_decode_default_split.argtypes = [fp, i32, i32, i32]
    lib.cq_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.cq_decode_workspace_bytes.argtypes = [fp, i32, i32, i32, i32]
    lib.cq_decode_attention.restype = ctypes.c_int
    lib.cq_decode_attention.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32,
                                        vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_decode_attention_static.restype = ctypes.c_int
    lib.cq_decode_attention_static.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32,
                                               vp, i32, vp, vp]
    lib.cq_decode_step.restype = ctypes.c_int
    lib.cq_decode_step.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32,
                                   vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_probe_stream_read.restype = ctypes.c_int
    lib.cq_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    pp = ctypes.POINTER(_PageTable)
    lib.cq_paged_cache_bytes.restype = ctypes.c_size_t
    lib.cq_paged_cache_bytes.argtypes = [fp, i32]
    lib.cq_encode_kv_paged.restype = ctypes.c_int
    lib.cq_encode_kv_paged.argtypes = [vp, vp, i64, i64, vp, vp, fp, i32, i32, vp, vp, pp, i32, vp]
    lib.cq_decode_attention_paged.restype = ctypes.c_int
    lib.cq_decode_attention_paged.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, pp, vp, i32, vp, vp,
                                              ctypes.c_size_t, vp]
    lib.cq_decode_step_paged.restype = ctypes.c_int
    lib.cq_decode_step_paged.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, pp, vp, i32,
                                         vp, vp, ctypes.c_size_t, vp]
    lib.cq_dequantize.restype = ctypes.c_int
    lib.cq_dequantize.argtypes = [vp, vp, fp, i32, i32, i32, i32, vp, i64, i64, vp]
    lib.cq_kmeans_workspace_bytes.restype = ctypes.c_size_t
    lib.cq_kmeans_workspace_bytes.argtypes = [fp, i32]
    lib.cq_kmeans_fit.restype = ctypes.c_int
    lib.cq_kmeans_fit.argtypes = [vp, i64, vp, fp, i32, i32, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.cq_fused_format.restype = ctypes.c_int
    lib.cq_fused_format.argtypes = [fp, fp]
    lib.cq_expand_codebook.restype = ctypes.c_int
    lib.cq_expand_codebook.argtypes = [vp, fp, vp, vp]
    lib.cq_chunk_default_split.restype = i32
    lib.cq_chunk_default_split.argtypes = [fp, i32, i32, i32, i32]
    lib.cq_chunk_workspace_bytes.restype = ctypes.c_size_t
    lib.cq_chunk_workspace_bytes.argtypes = [fp, i32, i32, i32, i32, i32]
    lib.cq_chunk_attention.restype = ctypes.c_int
    lib.cq_chunk_attention.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32, i32, vp, i32,
                                       vp, vp, ctypes.c_size_t, vp]
    lib.cq_chunk_attention_paged.restype = ctypes.c_int
    lib.cq_chunk_attention_paged.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32, pp, vp, i32,
                                             vp, vp, ctypes.c_size_t, vp]
    lib.cq_chunk_rope_workspace_bytes.restype = ctypes.c_size_t
    lib.cq_chunk_rope_workspace_bytes.argtypes = [fp, i32, i32, i32, i32, i32]
    lib.cq_chunk_attention_rope.restype = ctypes.c_int
    lib.cq_chunk_attention_rope.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32, i32, vp, i32,
                                            vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_chunk_attention_rope_paged.restype = ctypes.c_int
    lib.cq_chunk_attention_rope_paged.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32, pp, vp, i32,
                                                  vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_layer_table_bytes.restype = ctypes.c_size_t
    lib.cq_layer_table_bytes.argtypes = [i32]
    lib.cq_layer_table_fill.restype = ctypes.c_int
    lib.cq_layer_table_fill.argtypes = [ctypes.POINTER(_LayerIO), i32, vp, ctypes.c_size_t, vp]
    lib.cq_decode_step_layers.restype = ctypes.c_int
    lib.cq_decode_step_layers.argtypes = [vp, i32, i64, ctypes.c_float, fp, i32, i32, i32, i32, vp, i32, vp,
                                          ctypes.c_size_t, vp]
    lib.cq_rope_table_bytes.restype = ctypes.c_size_t
    lib.cq_rope_table_bytes.argtypes = [i32, i32]
    lib.cq_rope_table.restype = ctypes.c_int
    lib.cq_rope_table.argtypes = [ctypes.c_double, i32, i32, vp, ctypes.c_size_t, vp]
    lib.cq_decode_rope_default_split.restype = i32
    lib.cq_decode_rope_default_split.argtypes = [fp, i32, i32, i32]
    lib.cq_decode_attention_rope.restype = ctypes.c_int
    lib.cq_decode_attention_rope.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32,
                                             vp, i32, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_decode_attention_rope_paged.restype = ctypes.c_int
    lib.cq_decode_attention_rope_paged.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, pp, vp, i32,
                                                   vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_decode_step_rope.restype = ctypes.c_int
    lib.cq_decode_step_rope.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, i32,
                                        vp, i32, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_decode_step_rope_paged.restype = ctypes.c_int
    lib.cq_decode_step_rope_paged.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_float, fp, i32, i32, i32, pp, vp,
                                              i32, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.cq_probe_copy.restype = ctypes.c_int
    lib.cq_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.cq_probe_mfma.restype = ctypes.c_int
    lib.cq_probe_mfma.argtypes = [vp, vp, vp, i32, vp]
    _lib = lib
    return lib


def cq_version() -> int:
    return int(load().cq_version())


def status_string(status: int) -> str:
    return load().cq_status_string(int(status)).decode()


def cq_format_check(fmt: CQFormat) -> int:
    f = fmt._c()
    return int(load().cq_format_check(ctypes.byref(f)))


def cq_code_bytes_per_token_head(fmt: CQFormat) -> int:
    f = fmt._c()
    return int(load().cq_code_bytes_per_token_head(ctypes.byref(f)))


def cq_cache_bytes(fmt: CQFormat, batch: int, t_cap: int) -> int:
    f = fmt._c()
    return int(load().cq_cache_bytes(ctypes.byref(f), batch, t_cap))


def cq_decode_default_split(fmt: CQFormat, batch: int, n_q_heads: int, t: int) -> int:
    f = fmt._c()
    return int(load().cq_decode_default_split(ctypes.byref(f), batch, n_q_heads, t))


def cq_decode_workspace_bytes(fmt: CQFormat, batch: int, n_q_heads: int, t: int,
                              tokens_per_split: int = 0) -> int:
    f = fmt._c()
    return int(load().cq_decode_workspace_bytes(ctypes.byref(f), batch, n_q_heads, t, tokens_per_split))


def _stream_handle(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev(t, dtype, what: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must have dtype {dtype}, got {t.dtype}")
    return t


def alloc_cache(fmt: CQFormat, batch: int, t_cap: int, device="cuda"):
    """uint8 device buffer of cq_cache_bytes(fmt, batch, t_cap) bytes (uninitialised)."""
    import torch
    n = cq_cache_bytes(fmt, batch, t_cap)
    if n == 0:
        raise CQError(CQ_ERR_INVALID_ARG, "cq_cache_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


class PreparedCall:
    """An entry point with its arguments marshalled once: ``call()`` (or ``call(stream)``) only
    crosses the C ABI.  Keeps the tensors it points into alive."""
    __slots__ = ("_fn", "_args", "_keep", "_name")

    def __init__(self, fn, args, keep, name):
        self._fn, self._args, self._keep, self._name = fn, args, keep, name

    def __call__(self, stream=None):
        st = self._fn(*self._args, _stream_handle(stream))
        if st != CQ_OK:
            raise CQError(st, self._name)


def prepare_encode(x, centroids, fmt: CQFormat, codes, t_offset: int, t_cap: int) -> PreparedCall:
    """Check and marshal the arguments of cq_encode once (see cq_encode for their meaning)."""
    import torch
    _dev(x, torch.float16, "x")
    _dev(centroids, torch.float16, "centroids")
    _dev(codes, torch.uint8, "codes")
    if x.dim() != 3 or x.stride(2) != 1:
        raise ValueError("x must be [B, T_new, D] with a contiguous last dimension")
    if not centroids.is_contiguous() or not codes.is_contiguous():
        raise ValueError("centroids and codes must be contiguous")
    if tuple(centroids.shape) != (fmt.groups, 1 << fmt.b, fmt.c) or x.shape[2] != fmt.channels:
        raise ValueError("shapes do not match the format")
    batch, t_new = int(x.shape[0]), int(x.shape[1])
    if codes.numel() < cq_cache_bytes(fmt, batch, t_cap):
        raise ValueError("codes buffer is smaller than cq_cache_bytes(fmt, batch, t_cap)")
    f = fmt._c()
    args = (x.data_ptr(), x.stride(0), x.stride(1), centroids.data_ptr(), ctypes.byref(f),
            batch, t_new, codes.data_ptr(), t_offset, t_cap)
    return PreparedCall(load().cq_encode, args, (x, centroids, codes, f), "cq_encode")


def prepare_encode_kv(x_k, x_v, k_centroids, v_centroids, fmt: CQFormat, k_codes, v_codes, t_offset: int,
                      t_cap: int) -> PreparedCall:
    """Check and marshal the arguments of cq_encode_kv once (K and V in one launch)."""
    import torch
    for name, t in (("x_k", x_k), ("x_v", x_v), ("k_centroids", k_centroids), ("v_centroids", v_centroids)):
        _dev(t, torch.float16, name)
    _dev(k_codes, torch.uint8, "k_codes")
    _dev(v_codes, torch.uint8, "v_codes")
    if x_k.dim() != 3 or x_k.stride(2) != 1 or x_v.shape != x_k.shape or x_v.stride() != x_k.stride():
        raise ValueError("x_k and x_v must be [B, T_new, D] with equal shapes and strides")
    for cb in (k_centroids, v_centroids):
        if not cb.is_contiguous() or tuple(cb.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
            raise ValueError("centroids must be contiguous [G, 2^b, c]")
    if x_k.shape[2] != fmt.channels:
        raise ValueError("shapes do not match the format")
    batch, t_new = int(x_k.shape[0]), int(x_k.shape[1])
    need = cq_cache_bytes(fmt, batch, t_cap)
    if k_codes.numel() < need or v_codes.numel() < need:
        raise ValueError("code buffers are smaller than cq_cache_bytes(fmt, batch, t_cap)")
    f = fmt._c()
    args = (x_k.data_ptr(), x_v.data_ptr(), x_k.stride(0), x_k.stride(1), k_centroids.data_ptr(),
            v_centroids.data_ptr(), ctypes.byref(f), batch, t_new, k_codes.data_ptr(), v_codes.data_ptr(),
            t_offset, t_cap)
    keep = (x_k, x_v, k_centroids, v_centroids, k_codes, v_codes, f)
    return PreparedCall(load().cq_encode_kv, args, keep, "cq_encode_kv")


def cq_encode_kv(x_k, x_v, k_centroids, v_centroids, fmt: CQFormat, k_codes, v_codes, t_offset: int, t_cap: int,
                 stream=None) -> None:
    """cq_encode of a key and a value tensor of the same shape in one launch."""
    prepare_encode_kv(x_k, x_v, k_centroids, v_centroids, fmt, k_codes, v_codes, t_offset, t_cap)(stream)


def cq_encode(x, centroids, fmt: CQFormat, codes, t_offset: int, t_cap: int, stream=None) -> None:
    """x fp16 [B, T_new, D] (last dim contiguous), centroids fp16 [G, 2^b, c] contiguous,
    codes uint8 packed cache; writes the codes of the new tokens at positions t_offset..."""
    prepare_encode(x, centroids, fmt, codes, t_offset, t_cap)(stream)


def prepare_decode_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                             t: int, t_cap: int, seq_lens=None, tokens_per_split: int = 0,
                             out=None, workspace=None):
    """Check and marshal the arguments of cq_decode_attention once.  Returns (call, out)."""
    import torch
    _dev(q, torch.float16, "q")
    _dev(k_codes, torch.uint8, "k_codes")
    _dev(v_codes, torch.uint8, "v_codes")
    _dev(k_centroids, torch.float16, "k_centroids")
    _dev(v_centroids, torch.float16, "v_centroids")
    if q.dim() != 3 or not q.is_contiguous() or q.shape[2] != fmt.head_dim:
        raise ValueError("q must be contiguous [B, Hq, head_dim]")
    for name, cb in (("k_centroids", k_centroids), ("v_centroids", v_centroids)):
        if not cb.is_contiguous() or tuple(cb.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
            raise ValueError(f"{name} must be contiguous [G, 2^b, c]")
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    need_cache = cq_cache_bytes(fmt, batch, t_cap)
    if k_codes.numel() < need_cache or v_codes.numel() < need_cache:
        raise ValueError("code caches are smaller than cq_cache_bytes(fmt, batch, t_cap)")
    sl_ptr = None
    if seq_lens is not None:
        _dev(seq_lens, torch.int32, "seq_lens")
        if tuple(seq_lens.shape) != (batch,) or not seq_lens.is_contiguous():
            raise ValueError("seq_lens must be contiguous int32 [B]")
        sl_ptr = seq_lens.data_ptr()
    if out is None:
        out = torch.empty((batch, n_q_heads, fmt.head_dim), dtype=torch.float16, device=q.device)
    else:
        _dev(out, torch.float16, "out")
        if tuple(out.shape) != (batch, n_q_heads, fmt.head_dim) or not out.is_contiguous():
            raise ValueError("out must be contiguous [B, Hq, head_dim]")
    if workspace is None:
        nbytes = cq_decode_workspace_bytes(fmt, batch, n_q_heads, t, tokens_per_split)
        if nbytes == 0:
            raise CQError(CQ_ERR_INVALID_ARG, "cq_decode_workspace_bytes")
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    else:
        _dev(workspace, torch.uint8, "workspace")
    f = fmt._c()
    args = (q.data_ptr(), k_codes.data_ptr(), v_codes.data_ptr(), k_centroids.data_ptr(),
            v_centroids.data_ptr(), float(scale), ctypes.byref(f), batch, n_q_heads, t, t_cap, sl_ptr,
            tokens_per_split, out.data_ptr(), workspace.data_ptr(), workspace.numel())
    keep = (q, k_codes, v_codes, k_centroids, v_centroids, seq_lens, out, workspace, f)
    return PreparedCall(load().cq_decode_attention, args, keep, "cq_decode_attention"), out


STATIC_SCRATCH_BYTES = 4 << 20


def prepare_decode_attention_static(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                                    t: int, t_cap: int, out, seq_lens=None, tokens_per_split: int = 0):
    """Check and marshal the arguments of cq_decode_attention_static once (the caller brings
    `out`; nothing is allocated here or in the call).  Returns the call."""
    import torch
    _dev(q, torch.float16, "q")
    _dev(k_codes, torch.uint8, "k_codes")
    _dev(v_codes, torch.uint8, "v_codes")
    _dev(k_centroids, torch.float16, "k_centroids")
    _dev(v_centroids, torch.float16, "v_centroids")
    _dev(out, torch.float16, "out")
    if q.dim() != 3 or not q.is_contiguous() or q.shape[2] != fmt.head_dim:
        raise ValueError("q must be contiguous [B, Hq, head_dim]")
    for name, cb in (("k_centroids", k_centroids), ("v_centroids", v_centroids)):
        if not cb.is_contiguous() or tuple(cb.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
            raise ValueError(f"{name} must be contiguous [G, 2^b, c]")
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    need_cache = cq_cache_bytes(fmt, batch, t_cap)
    if k_codes.numel() < need_cache or v_codes.numel() < need_cache:
        raise ValueError("code caches are smaller than cq_cache_bytes(fmt, batch, t_cap)")
    if tuple(out.shape) != (batch, n_q_heads, fmt.head_dim) or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hq, head_dim]")
    sl_ptr = None
    if seq_lens is not None:
        _dev(seq_lens, torch.int32, "seq_lens")
        if tuple(seq_lens.shape) != (batch,) or not seq_lens.is_contiguous():
            raise ValueError("seq_lens must be contiguous int32 [B]")
        sl_ptr = seq_lens.data_ptr()
    f = fmt._c()
    args = (q.data_ptr(), k_codes.data_ptr(), v_codes.data_ptr(), k_centroids.data_ptr(),
            v_centroids.data_ptr(), float(scale), ctypes.byref(f), batch, n_q_heads, t, t_cap, sl_ptr,
            tokens_per_split, out.data_ptr())
    keep = (q, k_codes, v_codes, k_centroids, v_centroids, seq_lens, out, f)
    return PreparedCall(load().cq_decode_attention_static, args, keep, "cq_decode_attention_static")


def cq_decode_attention_static(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                               t: int, t_cap: int, out, seq_lens=None, tokens_per_split: int = 0, stream=None):
    """cq_decode_attention without a workspace (the library's static scratch array holds the
    partial results); `out` fp16 [B, Hq, head_dim] is the caller's."""
    prepare_decode_attention_static(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap, out,
                                    seq_lens, tokens_per_split)(stream)
    return out


def cq_decode_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                        t: int, t_cap: int, seq_lens=None, tokens_per_split: int = 0,
                        out=None, workspace=None, stream=None):
    """q fp16 [B, Hq, head_dim]; packed caches uint8; centroids fp16 [G, 2^b, c].  Returns out
    fp16 [B, Hq, head_dim] (allocated with torch if not given, as is the workspace)."""
    call, out = prepare_decode_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap,
                                         seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def cq_fused_format(fmt: CQFormat) -> CQFormat:
    """The format whose cache layout and decode kernels a format uses: itself for b = 8, 10,
    CQ-<c 8/b>c8b for the sub-byte formats b = 2, 4."""
    f, out = fmt._c(), _Format()
    st = load().cq_fused_format(ctypes.byref(f), ctypes.byref(out))
    if st != CQ_OK:
        raise CQError(st, "cq_fused_format")
    return CQFormat(out.c, out.b, out.head_dim, out.n_kv_heads)


def cq_expand_codebook(centroids, fmt: CQFormat, out=None, stream=None):
    """Sub-byte codebook fp16 [G, 2^b, c] -> the fused format's codebook fp16 [G b/8, 256, 8 c/b]."""
    import torch
    _dev(centroids, torch.float16, "centroids")
    if not centroids.is_contiguous() or tuple(centroids.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
        raise ValueError("centroids must be contiguous [G, 2^b, c]")
    fused = cq_fused_format(fmt)
    if out is None:
        out = torch.empty((fused.groups, 256, fused.c), dtype=torch.float16, device=centroids.device)
    _dev(out, torch.float16, "out")
    if not out.is_contiguous() or tuple(out.shape) != (fused.groups, 256, fused.c):
        raise ValueError("out must be contiguous [G b/8, 256, 8 c/b]")
    st = load().cq_expand_codebook(centroids.data_ptr(), ctypes.byref(fmt._c()), out.data_ptr(), _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_expand_codebook")
    return out


def cq_chunk_default_split(fmt: CQFormat, batch: int, n_q_heads: int, m: int, t: int) -> int:
    return int(load().cq_chunk_default_split(ctypes.byref(fmt._c()), batch, n_q_heads, m, t))


def cq_chunk_workspace_bytes(fmt: CQFormat, batch: int, n_q_heads: int, m: int, t: int, tokens_per_split: int = 0) -> int:
    return int(load().cq_chunk_workspace_bytes(ctypes.byref(fmt._c()), batch, n_q_heads, m, t, tokens_per_split))


def prepare_chunk_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int,
                            t_cap: int = 0, pages=None, seq_lens=None, tokens_per_split: int = 0, out=None,
                            workspace=None):
    """Check and marshal the arguments of cq_chunk_attention (or, with `pages`, of its paged form)
    once.  q fp16 [B, m, Hq, head_dim].  Returns (call, out)."""
    import torch
    _dev(q, torch.float16, "q")
    for name, x, dt in (("k_codes", k_codes, torch.uint8), ("v_codes", v_codes, torch.uint8),
                        ("k_centroids", k_centroids, torch.float16), ("v_centroids", v_centroids, torch.float16)):
        _dev(x, dt, name)
    if q.dim() != 4 or not q.is_contiguous() or q.shape[3] != fmt.head_dim:
        raise ValueError("q must be contiguous [B, m, Hq, head_dim]")
    for name, cb in (("k_centroids", k_centroids), ("v_centroids", v_centroids)):
        if not cb.is_contiguous() or tuple(cb.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
            raise ValueError(f"{name} must be contiguous [G, 2^b, c]")
    batch, m, n_q_heads = int(q.shape[0]), int(q.shape[1]), int(q.shape[2])
    need = cq_paged_cache_bytes(fmt, pages.n_pages) if pages is not None else cq_cache_bytes(fmt, batch, t_cap)
    if k_codes.numel() < need or v_codes.numel() < need:
        raise ValueError("code caches are smaller than the format, batch and capacity need")
    sl_ptr = None
    if seq_lens is not None:
        _dev(seq_lens, torch.int32, "seq_lens")
        if tuple(seq_lens.shape) != (batch,) or not seq_lens.is_contiguous():
            raise ValueError("seq_lens must be contiguous int32 [B]")
        sl_ptr = seq_lens.data_ptr()
    if out is None:
        out = torch.empty((batch, m, n_q_heads, fmt.head_dim), dtype=torch.float16, device=q.device)
    else:
        _dev(out, torch.float16, "out")
        if tuple(out.shape) != (batch, m, n_q_heads, fmt.head_dim) or not out.is_contiguous():
            raise ValueError("out must be contiguous [B, m, Hq, head_dim]")
    if workspace is None:
        workspace = torch.empty(max(16, cq_chunk_workspace_bytes(fmt, batch, n_q_heads, m, t, tokens_per_split)),
                                dtype=torch.uint8, device=q.device)
    else:
        _dev(workspace, torch.uint8, "workspace")
    f = fmt._c()
    head = (q.data_ptr(), k_codes.data_ptr(), v_codes.data_ptr(), k_centroids.data_ptr(), v_centroids.data_ptr(),
            float(scale), ctypes.byref(f), batch, n_q_heads, m, t)
    tail = (sl_ptr, tokens_per_split, out.data_ptr(), workspace.data_ptr(), workspace.numel())
    keep = (q, k_codes, v_codes, k_centroids, v_centroids, seq_lens, out, workspace, f, pages)
    if pages is not None:
        return PreparedCall(load().cq_chunk_attention_paged, head + (ctypes.byref(pages._c),) + tail, keep,
                            "cq_chunk_attention_paged"), out
    return PreparedCall(load().cq_chunk_attention, head + (t_cap,) + tail, keep, "cq_chunk_attention"), out


def cq_chunk_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int, t_cap: int,
                       seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None, stream=None):
    """Causal attention of the last m tokens of each sequence over its cache: q, out fp16
    [B, m, Hq, head_dim]; query j sits at position seq_len - m + j."""
    call, out = prepare_chunk_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap, None,
                                        seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def cq_chunk_attention_paged(q, k_pool, v_pool, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int, pages,
                             seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None, stream=None):
    """cq_chunk_attention over paged pools."""
    call, out = prepare_chunk_attention(q, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, t, 0, pages,
                                        seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


class LayerTable:
    """The device table of cq_layer_table_fill.  `layers`: one dict per layer with the tensors
    q [B, Hq, head_dim], x_k_new / x_v_new [B, D], k_codes, v_codes, k_centroids, v_centroids and
    out [B, Hq, head_dim] (as for cq_decode_step; all layers share shapes and the row stride)."""
    FIELDS = ("q", "x_k_new", "x_v_new", "k_codes", "v_codes", "k_centroids", "v_centroids", "out")

    def __init__(self, layers, fmt: CQFormat, t_cap: int, stream=None):
        import torch
        if not layers:
            raise ValueError("at least one layer")
        dtypes = dict(q=torch.float16, x_k_new=torch.float16, x_v_new=torch.float16, k_codes=torch.uint8,
                      v_codes=torch.uint8, k_centroids=torch.float16, v_centroids=torch.float16, out=torch.float16)
        first = layers[0]
        batch, n_q_heads = int(first["q"].shape[0]), int(first["q"].shape[1])
        need_cache = cq_cache_bytes(fmt, batch, t_cap)
        rec = (_LayerIO * len(layers))()
        for i, lay in enumerate(layers):
            for name in self.FIELDS:
                _dev(lay[name], dtypes[name], name)
            if tuple(lay["q"].shape) != (batch, n_q_heads, fmt.head_dim) or not lay["q"].is_contiguous():
                raise ValueError("q must be contiguous [B, Hq, head_dim], the same shape in every layer")
            if tuple(lay["out"].shape) != (batch, n_q_heads, fmt.head_dim) or not lay["out"].is_contiguous():
                raise ValueError("out must be contiguous [B, Hq, head_dim]")
            for name in ("x_k_new", "x_v_new"):
                x = lay[name]
                if tuple(x.shape) != (batch, fmt.channels) or x.stride(1) != 1 or x.stride(0) != first["x_k_new"].stride(0):
                    raise ValueError(f"{name} must be [B, D] with unit channel stride and one row stride for all layers")
            for name in ("k_centroids", "v_centroids"):
                if not lay[name].is_contiguous() or tuple(lay[name].shape) != (fmt.groups, 1 << fmt.b, fmt.c):
                    raise ValueError(f"{name} must be contiguous [G, 2^b, c]")
            for name in ("k_codes", "v_codes"):
                if lay[name].numel() < need_cache:
                    raise ValueError(f"{name} is smaller than cq_cache_bytes(fmt, batch, t_cap)")
            for j, name in enumerate(self.FIELDS):
                setattr(rec[i], name, lay[name].data_ptr())
        self.n_layers, self.batch, self.n_q_heads, self.t_cap, self.fmt = len(layers), batch, n_q_heads, int(t_cap), fmt
        self.x_row_stride = int(first["x_k_new"].stride(0))
        self._keep = [dict(lay) for lay in layers]
        nbytes = int(load().cq_layer_table_bytes(self.n_layers))
        self.table = torch.empty(nbytes, dtype=torch.uint8, device=first["q"].device)
        st = load().cq_layer_table_fill(rec, self.n_layers, self.table.data_ptr(), nbytes, _stream_handle(stream))
        if st != CQ_OK:
            raise CQError(st, "cq_layer_table_fill")

    def outputs(self):
        return [lay["out"] for lay in self._keep]


def prepare_decode_step_layers(table: LayerTable, scale: float, t: int, seq_lens=None, tokens_per_split: int = 0,
                               workspace=None) -> PreparedCall:
    """Check and marshal the arguments of cq_decode_step_layers once."""
    import torch
    if not isinstance(table, LayerTable):
        raise TypeError("table must be a LayerTable")
    fmt = table.fmt
    sl_ptr = None
    if seq_lens is not None:
        _dev(seq_lens, torch.int32, "seq_lens")
        if tuple(seq_lens.shape) != (table.batch,) or not seq_lens.is_contiguous():
            raise ValueError("seq_lens must be contiguous int32 [B]")
        sl_ptr = seq_lens.data_ptr()
    if workspace is None:
        nbytes = cq_decode_workspace_bytes(fmt, table.batch, table.n_q_heads, t, tokens_per_split)
        if nbytes == 0:
            raise CQError(CQ_ERR_INVALID_ARG, "cq_decode_workspace_bytes")
        workspace = torch.empty(nbytes * table.n_layers, dtype=torch.uint8, device=table.table.device)
    else:
        _dev(workspace, torch.uint8, "workspace")
    f = fmt._c()
    args = (table.table.data_ptr(), table.n_layers, table.x_row_stride, float(scale), ctypes.byref(f), table.batch,
            table.n_q_heads, t, table.t_cap, sl_ptr, tokens_per_split, workspace.data_ptr(), workspace.numel())
    return PreparedCall(load().cq_decode_step_layers, args, (table, seq_lens, workspace, f), "cq_decode_step_layers")


def cq_decode_step_layers(table: LayerTable, scale: float, t: int, seq_lens=None, tokens_per_split: int = 0,
                          workspace=None, stream=None):
    """cq_decode_step of every layer of the table in one launch; returns the layers' out tensors."""
    prepare_decode_step_layers(table, scale, t, seq_lens, tokens_per_split, workspace)(stream)
    return table.outputs()


class RopeTable:
    """The trigonometric table of cq_rope_table on the device: covers positions [0, positions)."""

    def __init__(self, base: float, positions: int, head_dim: int = 128, device="cuda", stream=None):
        import torch
        nbytes = int(load().cq_rope_table_bytes(head_dim, positions))
        if nbytes == 0:
            raise CQError(CQ_ERR_INVALID_ARG, "cq_rope_table_bytes")
        self.base, self.positions, self.head_dim = float(base), int(positions), int(head_dim)
        self.table = torch.empty(nbytes, dtype=torch.uint8, device=device)
        st = load().cq_rope_table(self.base, head_dim, positions, self.table.data_ptr(), nbytes, _stream_handle(stream))
        if st != CQ_OK:
            raise CQError(st, "cq_rope_table")


def cq_decode_rope_default_split(fmt: CQFormat, batch: int, n_q_heads: int, t: int) -> int:
    f = fmt._c()
    return int(load().cq_decode_rope_default_split(ctypes.byref(f), batch, n_q_heads, t))


def cq_chunk_rope_workspace_bytes(fmt: CQFormat, batch: int, n_q_heads: int, m: int, t: int, tokens_per_split: int = 0) -> int:
    f = fmt._c()
    return int(load().cq_chunk_rope_workspace_bytes(ctypes.byref(f), batch, n_q_heads, m, t, tokens_per_split))


def prepare_chunk_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int,
                                 t_cap: int, rope: "RopeTable", pages=None, seq_lens=None, tokens_per_split: int = 0,
                                 out=None, workspace=None):
    """Check and marshal the arguments of cq_chunk_attention_rope (or, with `pages`, of its paged
    form) once.  q fp16 [B, m, Hq, head_dim], each query token rotated to its own position.
    Returns (call, out)."""
    import torch
    if not isinstance(rope, RopeTable):
        raise TypeError("rope must be a RopeTable")
    batch, m, n_q_heads = int(q.shape[0]), int(q.shape[1]), int(q.shape[2])
    if workspace is None:
        nbytes = cq_chunk_rope_workspace_bytes(fmt, batch, n_q_heads, m, t, tokens_per_split)
        if nbytes == 0:
            raise CQError(CQ_ERR_INVALID_ARG, "cq_chunk_rope_workspace_bytes")
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    # the argument checks and the marshalling of the position-independent form, then the table
    call, out = prepare_chunk_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap, pages,
                                        seq_lens, tokens_per_split, out, workspace)
    a = call._args
    args = a[:-3] + (rope.table.data_ptr(), rope.positions) + a[-3:]
    name = "cq_chunk_attention_rope_paged" if pages is not None else "cq_chunk_attention_rope"
    return PreparedCall(getattr(load(), name), args, call._keep + (rope,), name), out


def cq_chunk_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int, t_cap: int,
                            rope: "RopeTable", seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None, stream=None):
    """cq_chunk_attention for caches whose keys were quantized before RoPE (token by token through
    the kernel of cq_decode_attention_rope): q, out fp16 [B, m, Hq, head_dim]."""
    call, out = prepare_chunk_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap, rope,
                                             None, seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def cq_chunk_attention_rope_paged(q, k_pool, v_pool, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int, pages,
                                  rope: "RopeTable", seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None,
                                  stream=None):
    """cq_chunk_attention_rope over paged pools."""
    call, out = prepare_chunk_attention_rope(q, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, t, 0, rope, pages,
                                             seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def prepare_decode_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                                  t: int, t_cap: int, rope: RopeTable, seq_lens=None, tokens_per_split: int = 0,
                                  out=None, workspace=None):
    """Check and marshal the arguments of cq_decode_attention_rope once.  Returns (call, out)."""
    if not isinstance(rope, RopeTable):
        raise TypeError("rope must be a RopeTable")
    if tokens_per_split == 0:
        tokens_per_split = cq_decode_rope_default_split(fmt, int(q.shape[0]), int(q.shape[1]), t)
        if tokens_per_split == 0:
            raise CQError(CQ_ERR_UNSUPPORTED, "cq_decode_rope_default_split")
    call, out = prepare_decode_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap,
                                         seq_lens, tokens_per_split, out, workspace)
    a = call._args
    args = a[:13] + (rope.table.data_ptr(), rope.positions) + a[13:]
    return PreparedCall(load().cq_decode_attention_rope, args, call._keep + (rope,), "cq_decode_attention_rope"), out


def cq_decode_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                             t: int, t_cap: int, rope: RopeTable, seq_lens=None, tokens_per_split: int = 0,
                             out=None, workspace=None, stream=None):
    """Decode attention over keys that were quantized before the rotary position embedding: q is
    already rotated to its position, the key of token u is rotated to position u on the fly."""
    call, out = prepare_decode_attention_rope(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap,
                                              rope, seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def prepare_decode_step_rope(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale: float,
                             fmt: CQFormat, t: int, t_cap: int, rope: RopeTable, seq_lens=None,
                             tokens_per_split: int = 0, out=None, workspace=None):
    """Check and marshal the arguments of cq_decode_step_rope once.  Returns (call, out)."""
    if not isinstance(rope, RopeTable):
        raise TypeError("rope must be a RopeTable")
    if tokens_per_split == 0:
        tokens_per_split = cq_decode_rope_default_split(fmt, int(q.shape[0]), int(q.shape[1]), t)
        if tokens_per_split == 0:
            raise CQError(CQ_ERR_UNSUPPORTED, "cq_decode_rope_default_split")
    call, out = prepare_decode_step(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t,
                                    t_cap, seq_lens, tokens_per_split, out, workspace)
    a = call._args
    args = a[:16] + (rope.table.data_ptr(), rope.positions) + a[16:]
    return PreparedCall(load().cq_decode_step_rope, args, call._keep + (rope,), "cq_decode_step_rope"), out


def cq_decode_step_rope(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                        t: int, t_cap: int, rope: RopeTable, seq_lens=None, tokens_per_split: int = 0, out=None,
                        workspace=None, stream=None):
    """cq_decode_step for caches of pre-rotation keys: x_k_new is the new key row BEFORE RoPE."""
    call, out = prepare_decode_step_rope(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale, fmt,
                                         t, t_cap, rope, seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def prepare_decode_step(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale: float,
                        fmt: CQFormat, t: int, t_cap: int, seq_lens=None, tokens_per_split: int = 0,
                        out=None, workspace=None):
    """Check and marshal the arguments of cq_decode_step once.  x_k_new / x_v_new: fp16 [B, D] (rows
    contiguous).  Returns (call, out)."""
    import torch
    call, out = prepare_decode_attention(q, k_codes, v_codes, k_centroids, v_centroids, scale, fmt, t, t_cap,
                                         seq_lens, tokens_per_split, out, workspace)
    batch = int(q.shape[0])
    for name, x in (("x_k_new", x_k_new), ("x_v_new", x_v_new)):
        _dev(x, torch.float16, name)
        if x.dim() != 2 or tuple(x.shape) != (batch, fmt.channels) or x.stride(1) != 1:
            raise ValueError(f"{name} must be [B, D] with contiguous rows")
    if x_k_new.stride(0) != x_v_new.stride(0):
        raise ValueError("x_k_new and x_v_new must have the same row stride")
    a = call._args
    args = (a[0], x_k_new.data_ptr(), x_v_new.data_ptr(), x_k_new.stride(0)) + a[1:]
    keep = call._keep + (x_k_new, x_v_new)
    return PreparedCall(load().cq_decode_step, args, keep, "cq_decode_step"), out


def cq_decode_step(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                   t: int, t_cap: int, seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None,
                   stream=None):
    """Fused cq_encode_kv of one new token per sequence (written at position t - 1, or
    seq_lens[n] - 1) + cq_decode_attention over t tokens.  Returns out fp16 [B, Hq, head_dim]."""
    call, out = prepare_decode_step(q, x_k_new, x_v_new, k_codes, v_codes, k_centroids, v_centroids, scale, fmt,
                                    t, t_cap, seq_lens, tokens_per_split, out, workspace)
    call(stream)
    return out


def cq_probe_stream_read(src, sink, stream=None) -> None:
    """Read every byte of the uint8 device tensor `src` once (measurement aid)."""
    import torch
    _dev(src, torch.uint8, "src")
    _dev(sink, torch.uint8, "sink")
    if sink.numel() < 8192:
        raise ValueError("sink must hold at least 8 KiB")
    st = load().cq_probe_stream_read(src.data_ptr(), src.numel(), sink.data_ptr(), _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_probe_stream_read")


def cq_probe_copy(src, dst, stream=None) -> None:
    """dst[:] = src for uint8 device tensors of equal size (measurement aid)."""
    import torch
    _dev(src, torch.uint8, "src")
    _dev(dst, torch.uint8, "dst")
    if dst.numel() != src.numel():
        raise ValueError("src and dst must have the same size")
    st = load().cq_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_probe_copy")


class PageTable:
    """A paged cache's block table: int32 device tensor [batch, max_tiles] (page of each 64-token
    tile of each sequence) over pools of n_pages pages."""

    def __init__(self, block_table, n_pages: int):
        import torch
        _dev(block_table, torch.int32, "block_table")
        if block_table.dim() != 2 or block_table.stride(1) != 1:
            raise ValueError("block_table must be [batch, max_tiles] with unit stride along tiles")
        self.block_table = block_table
        self.n_pages = int(n_pages)
        self._c = _PageTable(self.n_pages, int(block_table.shape[1]), int(block_table.stride(0)), block_table.data_ptr())

    @property
    def max_tiles(self) -> int:
        return int(self.block_table.shape[1])


def cq_paged_cache_bytes(fmt: CQFormat, n_pages: int) -> int:
    n = load().cq_paged_cache_bytes(ctypes.byref(fmt._c()), n_pages)
    if n == 0:
        raise CQError(CQ_ERR_INVALID_ARG, "cq_paged_cache_bytes")
    return n


def _check_centroids(fmt: CQFormat, k_centroids, v_centroids) -> None:
    import torch
    for name, cb in (("k_centroids", k_centroids), ("v_centroids", v_centroids)):
        _dev(cb, torch.float16, name)
        if not cb.is_contiguous() or tuple(cb.shape) != (fmt.groups, 1 << fmt.b, fmt.c):
            raise ValueError(f"{name} must be contiguous [G, 2^b, c]")


def cq_encode_kv_paged(x_k, x_v, k_centroids, v_centroids, fmt: CQFormat, k_pool, v_pool, pages: PageTable,
                       t_offset: int, stream=None) -> None:
    """cq_encode_kv into paged pools: x fp16 [B, T_new, D]; tokens go to positions t_offset ... of
    each sequence, i.e. to the pages pages.block_table names."""
    import torch
    for name, x in (("x_k", x_k), ("x_v", x_v)):
        _dev(x, torch.float16, name)
        if x.dim() != 3 or x.stride(2) != 1 or x.shape[2] != fmt.channels:
            raise ValueError(f"{name} must be [B, T_new, D] with unit channel stride")
    if x_k.shape != x_v.shape or x_k.stride() != x_v.stride():
        raise ValueError("x_k and x_v must have the same shape and strides")
    _check_centroids(fmt, k_centroids, v_centroids)
    need = cq_paged_cache_bytes(fmt, pages.n_pages)
    for name, t in (("k_pool", k_pool), ("v_pool", v_pool)):
        _dev(t, torch.uint8, name)
        if t.numel() < need:
            raise ValueError(f"{name} is smaller than cq_paged_cache_bytes(fmt, n_pages)")
    if pages.block_table.shape[0] < x_k.shape[0]:
        raise ValueError("block table has fewer rows than the batch")
    st = load().cq_encode_kv_paged(x_k.data_ptr(), x_v.data_ptr(), x_k.stride(0), x_k.stride(1), k_centroids.data_ptr(),
                                   v_centroids.data_ptr(), ctypes.byref(fmt._c()), int(x_k.shape[0]), int(x_k.shape[1]),
                                   k_pool.data_ptr(), v_pool.data_ptr(), ctypes.byref(pages._c), t_offset,
                                   _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_encode_kv_paged")


def _paged_decode(fn_name, q, x_k_new, x_v_new, k_pool, v_pool, k_centroids, v_centroids, scale, fmt, t, pages, seq_lens,
                  tokens_per_split, out, workspace, stream, rope=None):
    import torch
    _dev(q, torch.float16, "q")
    if q.dim() != 3 or not q.is_contiguous() or q.shape[2] != fmt.head_dim:
        raise ValueError("q must be contiguous [B, Hq, head_dim]")
    batch, n_q_heads = int(q.shape[0]), int(q.shape[1])
    _check_centroids(fmt, k_centroids, v_centroids)
    need = cq_paged_cache_bytes(fmt, pages.n_pages)
    for name, p in (("k_pool", k_pool), ("v_pool", v_pool)):
        _dev(p, torch.uint8, name)
        if p.numel() < need:
            raise ValueError(f"{name} is smaller than cq_paged_cache_bytes(fmt, n_pages)")
    if pages.block_table.shape[0] < batch:
        raise ValueError("block table has fewer rows than the batch")
    sl_ptr = None
    if seq_lens is not None:
        _dev(seq_lens, torch.int32, "seq_lens")
        sl_ptr = seq_lens.data_ptr()
    if out is None:
        out = torch.empty((batch, n_q_heads, fmt.head_dim), dtype=torch.float16, device=q.device)
    if workspace is None:
        workspace = torch.empty(max(16, cq_decode_workspace_bytes(fmt, batch, n_q_heads, t, tokens_per_split)),
                                dtype=torch.uint8, device=q.device)
    common = (k_pool.data_ptr(), v_pool.data_ptr(), k_centroids.data_ptr(), v_centroids.data_ptr(), float(scale),
              ctypes.byref(fmt._c()), batch, n_q_heads, t, ctypes.byref(pages._c), sl_ptr, tokens_per_split,
              out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream_handle(stream))
    if rope is not None and x_k_new is None:
        st = load().cq_decode_attention_rope_paged(q.data_ptr(), *common[:12], rope.table.data_ptr(), rope.positions,
                                                   *common[12:])
    elif x_k_new is None:
        st = load().cq_decode_attention_paged(q.data_ptr(), *common)
    else:
        for name, x in (("x_k_new", x_k_new), ("x_v_new", x_v_new)):
            _dev(x, torch.float16, name)
            if tuple(x.shape) != (batch, fmt.channels) or x.stride(1) != 1:
                raise ValueError(f"{name} must be [B, D] with unit channel stride")
        if x_k_new.stride(0) != x_v_new.stride(0):
            raise ValueError("x_k_new and x_v_new must share their row stride")
        if rope is not None:
            st = load().cq_decode_step_rope_paged(q.data_ptr(), x_k_new.data_ptr(), x_v_new.data_ptr(), x_k_new.stride(0),
                                                  *common[:12], rope.table.data_ptr(), rope.positions, *common[12:])
        else:
            st = load().cq_decode_step_paged(q.data_ptr(), x_k_new.data_ptr(), x_v_new.data_ptr(), x_k_new.stride(0), *common)
    if st != CQ_OK:
        raise CQError(st, fn_name)
    return out


def cq_decode_attention_paged(q, k_pool, v_pool, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int,
                              pages: PageTable, seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None,
                              stream=None):
    """cq_decode_attention over paged pools."""
    return _paged_decode("cq_decode_attention_paged", q, None, None, k_pool, v_pool, k_centroids, v_centroids, scale, fmt,
                         t, pages, seq_lens, tokens_per_split, out, workspace, stream)


def cq_decode_attention_rope_paged(q, k_pool, v_pool, k_centroids, v_centroids, scale: float, fmt: CQFormat, t: int,
                                   pages: PageTable, rope: RopeTable, seq_lens=None, tokens_per_split: int = 0,
                                   out=None, workspace=None, stream=None):
    """cq_decode_attention_rope over paged pools."""
    if tokens_per_split == 0:
        tokens_per_split = cq_decode_rope_default_split(fmt, int(q.shape[0]), int(q.shape[1]), t)
    return _paged_decode("cq_decode_attention_rope_paged", q, None, None, k_pool, v_pool, k_centroids, v_centroids,
                         scale, fmt, t, pages, seq_lens, tokens_per_split, out, workspace, stream, rope=rope)


def cq_decode_step_rope_paged(q, x_k_new, x_v_new, k_pool, v_pool, k_centroids, v_centroids, scale: float,
                              fmt: CQFormat, t: int, pages: PageTable, rope: RopeTable, seq_lens=None,
                              tokens_per_split: int = 0, out=None, workspace=None, stream=None):
    """cq_decode_step_rope over paged pools."""
    if tokens_per_split == 0:
        tokens_per_split = cq_decode_rope_default_split(fmt, int(q.shape[0]), int(q.shape[1]), t)
    return _paged_decode("cq_decode_step_rope_paged", q, x_k_new, x_v_new, k_pool, v_pool, k_centroids, v_centroids,
                         scale, fmt, t, pages, seq_lens, tokens_per_split, out, workspace, stream, rope=rope)


def cq_decode_step_paged(q, x_k_new, x_v_new, k_pool, v_pool, k_centroids, v_centroids, scale: float, fmt: CQFormat,
                         t: int, pages: PageTable, seq_lens=None, tokens_per_split: int = 0, out=None, workspace=None,
                         stream=None):
    """cq_decode_step over paged pools (the new token's codes go to the page of position t - 1)."""
    return _paged_decode("cq_decode_step_paged", q, x_k_new, x_v_new, k_pool, v_pool, k_centroids, v_centroids, scale,
                         fmt, t, pages, seq_lens, tokens_per_split, out, workspace, stream)


def cq_dequantize(codes, centroids, fmt: CQFormat, batch: int, t_offset: int, t_count: int, t_cap: int, out=None,
                  stream=None):
    """fp16 [batch, t_count, D] = the centroids the cached codes of positions t_offset .. t_offset +
    t_count - 1 select (out may be a strided view with unit channel stride)."""
    import torch
    _dev(codes, torch.uint8, "codes")
    _dev(centroids, torch.float16, "centroids")
    D = fmt.channels
    if out is None:
        out = torch.empty((batch, t_count, D), dtype=torch.float16, device=codes.device)
    _dev(out, torch.float16, "out")
    if tuple(out.shape) != (batch, t_count, D) or out.stride(2) != 1:
        raise ValueError("out must be [batch, t_count, D] with unit channel stride")
    st = load().cq_dequantize(codes.data_ptr(), centroids.data_ptr(), ctypes.byref(fmt._c()), batch, t_offset, t_count,
                              t_cap, out.data_ptr(), out.stride(0), out.stride(1), _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_dequantize")
    return out


KMEANS_MAX_POINTS = 524288


def cq_kmeans_workspace_bytes(fmt: CQFormat, n_points: int) -> int:
    n = load().cq_kmeans_workspace_bytes(ctypes.byref(fmt._c()), n_points)
    if n == 0:
        raise CQError(CQ_ERR_INVALID_ARG, "cq_kmeans_workspace_bytes")
    return n


def cq_kmeans_fit(x, fmt: CQFormat, n_iter: int, rnd=None, init_centroids=None, weights=None,
                  want_picks: bool = False, want_assignment: bool = False, workspace=None, stream=None) -> dict:
    """Centroid learning for every channel group of x fp16 [n, D] (device): k-means++ from the
    random words rnd uint64-as-int64 [G, 2^b] (or the given fp32 init_centroids [G, 2^b, c]), then
    n_iter Lloyd iterations, optionally weighted by weights fp32 [n, G].  Returns a dict with
    "centroids" (fp16 [G, 2^b, c]), "centroids_f32", and on request "picks" (int32 [G, 2^b]) and
    "assignment" (int16 view of uint16 [G, n])."""
    import torch
    _dev(x, torch.float16, "x")
    if x.dim() != 2 or x.shape[1] != fmt.n_kv_heads * fmt.head_dim or x.stride(1) != 1:
        raise ValueError("x must be [n, D] with unit channel stride")
    n = x.shape[0]
    G, K, c = fmt.groups, 1 << fmt.b, fmt.c
    dev = x.device
    if rnd is not None:
        _dev(rnd, torch.int64, "rnd")
        if tuple(rnd.shape) != (G, K) or not rnd.is_contiguous():
            raise ValueError("rnd must be a contiguous int64 tensor [G, 2^b] holding the 64-bit random words")
    if init_centroids is not None:
        _dev(init_centroids, torch.float32, "init_centroids")
        if tuple(init_centroids.shape) != (G, K, c) or not init_centroids.is_contiguous():
            raise ValueError("init_centroids must be contiguous fp32 [G, 2^b, c]")
    if weights is not None:
        _dev(weights, torch.float32, "weights")
        if tuple(weights.shape) != (n, G) or not weights.is_contiguous():
            raise ValueError("weights must be contiguous fp32 [n, G]")
    need = cq_kmeans_workspace_bytes(fmt, n)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _dev(workspace, torch.uint8, "workspace")
    cent16 = torch.empty((G, K, c), dtype=torch.float16, device=dev)
    cent32 = torch.empty((G, K, c), dtype=torch.float32, device=dev)
    picks = torch.empty((G, K), dtype=torch.int32, device=dev) if want_picks else None
    assign = torch.empty((G, n), dtype=torch.int16, device=dev) if want_assignment else None
    ptr = lambda t: None if t is None else t.data_ptr()
    st = load().cq_kmeans_fit(x.data_ptr(), x.stride(0), ptr(weights), ctypes.byref(fmt._c()), n, n_iter, ptr(rnd),
                              ptr(init_centroids), ptr(picks), cent16.data_ptr(), cent32.data_ptr(), ptr(assign),
                              workspace.data_ptr(), workspace.numel(), _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_kmeans_fit")
    out = {"centroids": cent16, "centroids_f32": cent32}
    if want_picks:
        out["picks"] = picks
    if want_assignment:
        out["assignment"] = assign
    return out


def cq_probe_mfma(a, b, stream=None):
    """D = A B by one matrix-core instruction: a fp16 [32, kdim], b fp16 [kdim, 32] (kdim 8 or 16,
    contiguous device tensors) -> fp32 [32, 32] (measurement aid)."""
    import torch
    _dev(a, torch.float16, "a")
    _dev(b, torch.float16, "b")
    kdim = a.shape[1]
    if tuple(a.shape) != (32, kdim) or tuple(b.shape) != (kdim, 32) or not (a.is_contiguous() and b.is_contiguous()):
        raise ValueError("a must be [32, kdim] and b [kdim, 32], contiguous")
    d = torch.empty((32, 32), dtype=torch.float32, device=a.device)
    st = load().cq_probe_mfma(a.data_ptr(), b.data_ptr(), d.data_ptr(), kdim, _stream_handle(stream))
    if st != CQ_OK:
        raise CQError(st, "cq_probe_mfma")
    return d
