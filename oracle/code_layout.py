"""numpy pack / unpack of the packed code cache.

TEST INFRASTRUCTURE: an independent statement, in numpy, of the cache layout
that the library documents in its public header.  The paper fixes only the
density of the stored codes (bits per floating-point number = b / c,
Section 4 "Baselines" paragraph and the "Bits Per FPN" column of Table 1);
the arrangement of the bits is this project's and is restated here:

* one stream per (sequence n, KV head h); streams are laid out ``[n][h]``;
* a stream is a sequence of tiles of 64 tokens; ``t_cap`` (a multiple of 64)
  tokens are reserved per stream; a tile takes ``64 * Gh * b / 8`` bytes,
  ``Gh = head_dim / c`` being the number of channel groups of one head;
* b = 8: the tile is ``Gh / 16`` planes of ``64 x 16`` bytes; byte ``w`` of token
  ``u``'s 16 bytes in plane ``p`` is *slot* ``s = 16 p + w`` and holds the code of
  group ``(s + u) mod Gh`` of that head (a per-token rotation of the groups);
* b = 10 (Gh = 16): a ``64 x 16``-byte plane with the low 8 bits of the code in
  each slot (same rotation), followed by a ``64 x 4``-byte plane holding, per
  token, a little-endian uint32 whose bits ``[2 s + 1 : 2 s]`` are the high two
  bits of the code in slot ``s``.

The logical object is ``codes[n, t, g]`` (uint16, ``g`` over all ``Hkv * Gh``
groups, head-major).
"""
from __future__ import annotations

import numpy as np

TILE_TOKENS = 64


def groups_per_head(c: int, head_dim: int) -> int:
    if head_dim % c:
        raise ValueError("c must divide head_dim")
    return head_dim // c


def bytes_per_token_head(c: int, b: int, head_dim: int) -> int:
    bits = groups_per_head(c, head_dim) * b
    if bits % 8:
        raise ValueError("a token-head's codes must fill whole bytes")
    return bits // 8


def tile_bytes(c: int, b: int, head_dim: int) -> int:
    return TILE_TOKENS * bytes_per_token_head(c, b, head_dim)


def cache_bytes(c: int, b: int, head_dim: int, n_kv_heads: int, batch: int, t_cap: int) -> int:
    if t_cap % TILE_TOKENS:
        raise ValueError("t_cap must be a multiple of 64")
    return batch * n_kv_heads * (t_cap // TILE_TOKENS) * tile_bytes(c, b, head_dim)


def bits_per_fpn(c: int, b: int, head_dim: int) -> float:
    """Stored code bits of one token-head divided by its number of fp values."""
    return 8.0 * bytes_per_token_head(c, b, head_dim) / head_dim


def pack(codes: np.ndarray, c: int, b: int, head_dim: int, n_kv_heads: int, t_cap: int,
         t_offset: int = 0, into: np.ndarray | None = None, fill: int = 0) -> np.ndarray:
    """codes uint16 [B, T, G] -> uint8 [B, Hkv, t_cap/64, tile_bytes], tokens placed at
    positions t_offset .. t_offset+T-1.  ``into`` updates an existing cache in place."""
    if b not in (8, 10):
        raise ValueError("only b = 8 and b = 10 have a layout")
    codes = np.asarray(codes)
    B, T, G = codes.shape
    Gh = groups_per_head(c, head_dim)
    if G != Gh * n_kv_heads:
        raise ValueError("G does not match the format")
    if b == 10 and Gh != 16:
        raise ValueError("the 10-bit layout is defined for 16 groups per head")
    if Gh % 16 or TILE_TOKENS % Gh:
        raise ValueError("groups per head must be 16, 32 or 64")
    if t_cap % TILE_TOKENS or t_offset < 0 or t_offset + T > t_cap:
        raise ValueError("token range does not fit the cache")
    if np.any(codes >= (1 << b)):
        raise ValueError("code out of range")
    tb = tile_bytes(c, b, head_dim)
    if into is None:
        cache = np.full((B, n_kv_heads, t_cap // TILE_TOKENS, tb), fill, dtype=np.uint8)
    else:
        cache = into
        if cache.shape != (B, n_kv_heads, t_cap // TILE_TOKENS, tb) or cache.dtype != np.uint8:
            raise ValueError("cache has the wrong shape")
    ch = codes.reshape(B, T, n_kv_heads, Gh).astype(np.uint32)
    t = np.arange(t_offset, t_offset + T)
    tile = t // TILE_TOKENS
    u = t % TILE_TOKENS
    n_planes = Gh // 16
    hi_word = np.zeros((B, n_kv_heads, T), dtype=np.uint32)
    for s in range(Gh):
        g = (s + u) % Gh                                     # [T]
        val = ch[:, np.arange(T), :, g]                      # [T, B, Hkv] (advanced indexing first)
        val = np.transpose(val, (1, 2, 0))                   # [B, Hkv, T]
        p, w = divmod(s, 16)
        cache[:, :, tile, p * 1024 + u * 16 + w] = (val & 0xFF).astype(np.uint8)
        if b == 10:
            hi_word |= (val >> 8) << np.uint32(2 * s)
    if b == 10:
        base = n_planes * 1024
        for k in range(4):
            cache[:, :, tile, base + u * 4 + k] = ((hi_word >> np.uint32(8 * k)) & 0xFF).astype(np.uint8)
    return cache


def unpack(cache: np.ndarray, c: int, b: int, head_dim: int, n_kv_heads: int,
           n_tokens: int, t_offset: int = 0) -> np.ndarray:
    """Inverse of ``pack``: uint8 [B, Hkv, t_cap/64, tile_bytes] -> uint16 [B, T, G]."""
    if b not in (8, 10):
        raise ValueError("only b = 8 and b = 10 have a layout")
    Gh = groups_per_head(c, head_dim)
    tb = tile_bytes(c, b, head_dim)
    B, H, n_tiles, tb2 = cache.shape
    if H != n_kv_heads or tb2 != tb:
        raise ValueError("cache has the wrong shape")
    T = n_tokens
    if t_offset + T > n_tiles * TILE_TOKENS:
        raise ValueError("token range exceeds the cache")
    t = np.arange(t_offset, t_offset + T)
    tile = t // TILE_TOKENS
    u = t % TILE_TOKENS
    out = np.zeros((B, T, n_kv_heads, Gh), dtype=np.uint16)
    n_planes = Gh // 16
    if b == 10:
        base = n_planes * 1024
        hi_word = np.zeros((B, H, T), dtype=np.uint32)
        for k in range(4):
            hi_word |= cache[:, :, tile, base + u * 4 + k].astype(np.uint32) << np.uint32(8 * k)
    for s in range(Gh):
        g = (s + u) % Gh
        p, w = divmod(s, 16)
        val = cache[:, :, tile, p * 1024 + u * 16 + w].astype(np.uint16)      # [B, H, T]
        if b == 10:
            val = val | (((hi_word >> np.uint32(2 * s)) & 3).astype(np.uint16) << 8)
        # out[n, t, h, g[t]] = val[n, h, t]
        out[:, np.arange(T), :, g] = np.transpose(val, (2, 0, 1))
    return out.reshape(B, T, n_kv_heads * Gh)
