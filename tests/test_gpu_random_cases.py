"""Randomly drawn (seeded) valid calls of every decode-side entry point against the CPU oracle:
format, head counts, grouped queries, batch, context, capacity, context split, ragged lengths,
paged pools and the entry point itself (attention, fused step, their pre-RoPE forms, several
query tokens with and without rotation) are drawn together, so that combinations no hand-written
case names still meet the oracle element by element."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O

from gpu_util import cache_to_codes, check_attention, check_codes, codes_to_cache, dev

pytestmark = pytest.mark.gpu

FORMATS = [(8, 8), (4, 8), (2, 8), (8, 10)]
MAX_TILES = {(8, 8): 1000, (4, 8): 1000, (2, 8): 128, (8, 10): 256}
MODES = ["attention", "step", "rope", "rope_step", "chunk", "rope_chunk"]
BASE = 10000.0


def _draw(i):
    rng = np.random.default_rng(2405_03917 + i)
    c, b = FORMATS[i % 4]
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    hq = hkv * int(rng.choice([1, 2, 4]))
    B = int(rng.integers(1, 4))
    T = int(rng.choice([1, 2, 63, 64, 65, 130, 500, 1100, int(rng.integers(1, 1500)), int(rng.integers(3000, 12000))]))
    mode = MODES[(i // 4) % len(MODES)]
    m = int(min(T, rng.integers(1, 7))) if "chunk" in mode else 1
    t_cap = -(-T // 64) * 64 + 64 * int(rng.integers(0, 3))
    max_tiles = min(MAX_TILES[(c, b)], 128) if "rope" in mode else MAX_TILES[(c, b)]
    tiles = -(-T // 64)
    split = 64 * int(rng.integers(1, min(tiles, max_tiles) + 1)) if rng.random() < 0.5 else 0
    if split and tiles * 64 // split > 64:
        split = 0                                   # (keeps the number of splits moderate)
    return dict(c=c, b=b, hq=hq, hkv=hkv, B=B, T=T, mode=mode, m=m, t_cap=t_cap, split=split,
                ragged=bool(rng.random() < 0.5), paged=bool(rng.random() < 0.4),
                scale=float(rng.choice([0.05, 1 / math.sqrt(128), 0.2])), seed=i)


def _pools(caches, fmt, B, t_cap, rng):
    n_tiles = t_cap // 64
    n_pages = B * n_tiles + int(rng.integers(0, 4))
    perm = rng.permutation(n_pages)[:B * n_tiles].astype(np.int32).reshape(B, n_tiles)
    tb = cq.cq_code_bytes_per_token_head(fmt) * 64
    pools = []
    for cache in caches:
        src = cache.cpu().numpy().reshape(B, fmt.n_kv_heads, n_tiles, tb)
        pool = np.full((n_pages, fmt.n_kv_heads, tb), 0x77, dtype=np.uint8)
        for n in range(B):
            for t in range(n_tiles):
                pool[perm[n, t]] = src[n, :, t]
        pools.append(dev(pool.reshape(-1)))
    return pools, cq.PageTable(dev(perm), n_pages), perm, n_pages


def _gather_pages(pool, fmt, B, t_cap, perm, n_pages):
    n_tiles = t_cap // 64
    tb = cq.cq_code_bytes_per_token_head(fmt) * 64
    pl = pool.cpu().numpy().reshape(n_pages, fmt.n_kv_heads, tb)
    out = np.empty((B, fmt.n_kv_heads, n_tiles, tb), dtype=np.uint8)
    for n in range(B):
        for t in range(n_tiles):
            out[n, :, t] = pl[perm[n, t]]
    return dev(out.reshape(-1))


@pytest.mark.parametrize("i", range(96))
def test_random_valid_call_matches_oracle(i):
    p = _draw(i)
    c, b, hq, hkv, B, T, m, t_cap, split, scale = (p[k] for k in ("c", "b", "hq", "hkv", "B", "T", "m", "t_cap", "split", "scale"))
    mode, paged = p["mode"], p["paged"]
    rng = np.random.default_rng(7000 + i)
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(200 + i, 0, "k", D), synth.tensor_recipe(200 + i, 0, "v", D)
    ck, cv = synth.sample_codebook(rk, c, b), synth.sample_codebook(rv, c, b)
    kc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    vc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    lens = rng.integers(m, T + 1, size=B).astype(np.int32) if p["ragged"] else None
    full = np.full(B, T, dtype=np.int32) if lens is None else lens
    sl = None if lens is None else dev(lens)
    rope = cq.RopeTable(BASE, t_cap) if "rope" in mode else None
    base = BASE if rope else None
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    if paged:
        pools, pages, perm, n_pages = _pools((kcache, vcache), fmt, B, t_cap, rng)
    dck, dcv = dev(ck), dev(cv)
    kw = dict(seq_lens=sl, tokens_per_split=split)

    if "chunk" in mode:
        q = rng.standard_normal((B, m, hq, 128)).astype(np.float16)
        ref = O.chunk_attention(q, kc, vc, ck, cv, scale, hkv, seq_lens=lens, rope_base=base)
        if mode == "chunk":
            out = (cq.cq_chunk_attention_paged(dev(q), pools[0], pools[1], dck, dcv, scale, fmt, T, pages, **kw) if paged
                   else cq.cq_chunk_attention(dev(q), kcache, vcache, dck, dcv, scale, fmt, T, t_cap, **kw))
        else:
            out = (cq.cq_chunk_attention_rope_paged(dev(q), pools[0], pools[1], dck, dcv, scale, fmt, T, pages, rope, **kw) if paged
                   else cq.cq_chunk_attention_rope(dev(q), kcache, vcache, dck, dcv, scale, fmt, T, t_cap, rope, **kw))
        torch.cuda.synchronize()
        check_attention(out.cpu().numpy().reshape(B * m, hq, 128), ref.reshape(B * m, hq, 128))
        return

    q = rng.standard_normal((B, hq, 128)).astype(np.float16)
    if "step" in mode:
        xk = np.concatenate([synth.sample_activations(rk, 1, chunk=900 + n) for n in range(B)])
        xv = np.concatenate([synth.sample_activations(rv, 1, chunk=950 + n) for n in range(B)])
        extra = (rope,) if rope else ()
        if paged:
            fn = cq.cq_decode_step_rope_paged if rope else cq.cq_decode_step_paged
            out = fn(dev(q), dev(xk), dev(xv), pools[0], pools[1], dck, dcv, scale, fmt, T, pages, *extra, **kw)
        else:
            fn = cq.cq_decode_step_rope if rope else cq.cq_decode_step
            out = fn(dev(q), dev(xk), dev(xv), kcache, vcache, dck, dcv, scale, fmt, T, t_cap, *extra, **kw)
        torch.cuda.synchronize()
        if paged:
            kcache, vcache = (_gather_pages(pl, fmt, B, t_cap, perm, n_pages) for pl in pools)
        kcodes, vcodes = cache_to_codes(kcache, fmt, B, t_cap, T), cache_to_codes(vcache, fmt, B, t_cap, T)
        for n in range(B):
            pos = int(full[n]) - 1                  # the new token's codes: the oracle's, up to near ties
            check_codes(kcodes[n, pos:pos + 1], xk[n:n + 1], ck)
            check_codes(vcodes[n, pos:pos + 1], xv[n:n + 1], cv)
            others = np.arange(T) != pos            # and no other token's codes were touched
            assert np.array_equal(kcodes[n, others], kc[n, others]) and np.array_equal(vcodes[n, others], vc[n, others])
        ref = O.attention(q, kcodes, vcodes, ck, cv, scale, hkv, seq_lens=lens, rope_base=base)
        check_attention(out.cpu().numpy(), ref)
        return

    ref = O.attention(q, kc, vc, ck, cv, scale, hkv, seq_lens=lens, rope_base=base)
    if paged:
        out = (cq.cq_decode_attention_rope_paged(dev(q), pools[0], pools[1], dck, dcv, scale, fmt, T, pages, rope, **kw) if rope
               else cq.cq_decode_attention_paged(dev(q), pools[0], pools[1], dck, dcv, scale, fmt, T, pages, **kw))
    else:
        out = (cq.cq_decode_attention_rope(dev(q), kcache, vcache, dck, dcv, scale, fmt, T, t_cap, rope, **kw) if rope
               else cq.cq_decode_attention(dev(q), kcache, vcache, dck, dcv, scale, fmt, T, t_cap, **kw))
    torch.cuda.synchronize()
    check_attention(out.cpu().numpy(), ref)


ENCODE_FORMATS = FORMATS + [(1, 2), (2, 2), (1, 4), (2, 4), (4, 4)]


@pytest.mark.parametrize("i", range(54))
def test_random_valid_encode_matches_oracle(i):
    """cq_encode / cq_encode_kv on strided inputs at random offsets, every format (the sub-byte
    ones through their fused byte codes): the oracle's codes up to near ties, and no byte of any
    other token touched."""
    rng = np.random.default_rng(9000 + i)
    c, b = ENCODE_FORMATS[i % len(ENCODE_FORMATS)]
    hkv = int(rng.choice([1, 2, 3, 8]))
    B = int(rng.integers(1, 4))
    t_new = int(rng.choice([1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 200, int(rng.integers(1, 700))]))
    t_off = int(rng.choice([0, 1, 63, 64, 100, int(rng.integers(0, 300))]))
    t_cap = -(-(t_off + t_new) // 64) * 64 + 64 * int(rng.integers(0, 2))
    both, pad, gap = bool(rng.random() < 0.5), int(rng.choice([0, 8, 64])), int(rng.choice([0, 3]))
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(300 + i, 0, "k", D), synth.tensor_recipe(300 + i, 0, "v", D)
    if b >= 8:
        ck, cv = synth.sample_codebook(rk, c, b), synth.sample_codebook(rv, c, b)
    else:
        ck = (rng.standard_normal((D // c, 1 << b, c)) * 1.5).astype(np.float16)
        cv = (rng.standard_normal((D // c, 1 << b, c)) * 1.5).astype(np.float16)
    xk = np.stack([synth.sample_activations(rk, t_new, chunk=n) for n in range(B)])
    xv = np.stack([synth.sample_activations(rv, t_new, chunk=50 + n) for n in range(B)])

    def strided(x):                                 # rows and sequences further apart than they need to be
        buf = torch.full((B, t_new + gap, D + pad), 7.0, dtype=torch.float16, device="cuda")
        buf[:, :t_new, :D] = dev(x)
        return buf[:, :t_new, :D]

    fill = 0xA5
    kcache = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), fill, dtype=torch.uint8, device="cuda")
    vcache = torch.full_like(kcache, fill)
    if both:
        cq.cq_encode_kv(strided(xk), strided(xv), dev(ck), dev(cv), fmt, kcache, vcache, t_off, t_cap)
    else:
        cq.cq_encode(strided(xk), dev(ck), fmt, kcache, t_off, t_cap)
        cq.cq_encode(strided(xv), dev(cv), fmt, vcache, t_off, t_cap)
    torch.cuda.synchronize()
    stored = fmt if b >= 8 else cq.cq_fused_format(fmt)         # the format of the bytes in the cache
    untouched = np.ones(t_cap, dtype=bool)
    untouched[t_off:t_off + t_new] = False
    blank = cache_to_codes(torch.full_like(kcache, fill), stored, B, t_cap, t_cap)
    for cache, x, cb in ((kcache, xk, ck), (vcache, xv, cv)):
        codes = cache_to_codes(cache, stored, B, t_cap, t_new, t_off)
        if b < 8:       # a byte holds the codes of 8 / b neighbouring groups, lowest group in the lowest bits
            fuse = 8 // b
            codes = np.stack([(codes >> (b * k)) & ((1 << b) - 1) for k in range(fuse)], axis=-1).reshape(B, t_new, -1)
        for n in range(B):
            check_codes(codes[n], x[n], cb)
        assert np.array_equal(cache_to_codes(cache, stored, B, t_cap, t_cap)[:, untouched], blank[:, untouched])
