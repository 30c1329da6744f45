"""Paged caches: the *_paged entry points on pools of shuffled pages must give exactly what the
contiguous entry points give on the same logical contents (which the other GPU tests tie to the
oracle), and leave pages that no sequence owns untouched."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O

from gpu_util import cache_to_codes, check_attention, dev

pytestmark = pytest.mark.gpu

FORMATS = [(8, 8), (4, 8), (2, 8), (8, 10)]


def _setup(seed, c, b, hkv, hq, B, T, extra_pages=5):
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(80 + seed, 0, "k", D), synth.tensor_recipe(80 + seed, 0, "v", D)
    xk = np.stack([synth.sample_activations(rk, T, chunk=n) for n in range(B)])
    xv = np.stack([synth.sample_activations(rv, T, chunk=n) for n in range(B)])
    ck, cv = synth.sample_codebook(rk, c, b), synth.sample_codebook(rv, c, b)
    q = np.random.default_rng(seed).standard_normal((B, hq, 128)).astype(np.float16)
    tiles = -(-T // 64)
    n_pages = B * tiles + extra_pages
    rng = np.random.default_rng(seed + 1)
    perm = rng.permutation(n_pages)
    table = perm[:B * tiles].reshape(B, tiles).astype(np.int32)
    wide = np.full((B, tiles + 3), -7, dtype=np.int32)           # row stride > max_tiles, junk beyond
    wide[:, :tiles] = table
    bt = dev(wide)[:, :tiles]
    return fmt, xk, xv, ck, cv, q, tiles, n_pages, perm, cq.PageTable(bt, n_pages)


def _pool_to_cache(pool, fmt, table, n_pages):
    """Gather a pool [page][hkv][tile bytes] into the contiguous layout [n][hkv][tile][tile bytes]."""
    tb = pool.numel() // (n_pages * fmt.n_kv_heads)
    p = pool.view(n_pages, fmt.n_kv_heads, tb)
    t = torch.from_numpy(table.astype(np.int64)).cuda()
    return p[t].permute(0, 2, 1, 3).contiguous().view(-1)           # [B, tiles, hkv, tb] -> [B, hkv, tiles, tb]


@pytest.mark.parametrize("c,b", FORMATS)
def test_paged_encode_and_decode_equal_the_contiguous_calls(c, b):
    hkv, hq, B, T = 2, 4, 3, 333
    fmt, xk, xv, ck, cv, q, tiles, n_pages, perm, pages = _setup(c + b, c, b, hkv, hq, B, T)
    t_cap = tiles * 64
    table = perm[:B * tiles].reshape(B, tiles)
    ckd, cvd, qd = dev(ck), dev(cv), dev(q)
    # contiguous reference
    kc = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), 0xA5, dtype=torch.uint8, device="cuda")
    vc = torch.full_like(kc, 0xA5)
    cq.cq_encode_kv(dev(xk), dev(xv), ckd, cvd, fmt, kc, vc, 0, t_cap)
    # paged, filled in two calls (a prefill and an append that straddles a page boundary)
    nbytes = cq.cq_paged_cache_bytes(fmt, n_pages)
    kp = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    vp = torch.full_like(kp, 0xA5)
    cut = 190
    cq.cq_encode_kv_paged(dev(xk[:, :cut]), dev(xv[:, :cut]), ckd, cvd, fmt, kp, vp, pages, 0)
    cq.cq_encode_kv_paged(dev(xk[:, cut:]), dev(xv[:, cut:]), ckd, cvd, fmt, kp, vp, pages, cut)
    torch.cuda.synchronize()
    assert torch.equal(_pool_to_cache(kp, fmt, table, n_pages), kc)
    assert torch.equal(_pool_to_cache(vp, fmt, table, n_pages), vc)
    tb = nbytes // (n_pages * hkv)
    unused = torch.from_numpy(perm[B * tiles:].astype(np.int64)).cuda()
    assert bool((kp.view(n_pages, hkv * tb)[unused] == 0xA5).all()) and bool((vp.view(n_pages, hkv * tb)[unused] == 0xA5).all())
    # decode attention: several splits, ragged lengths
    lens = np.array([T, 1, 130], dtype=np.int32)
    for split, sl in ((0, None), (64, dev(lens)), (192, dev(lens))):
        ref = cq.cq_decode_attention(qd, kc, vc, ckd, cvd, 0.09, fmt, T, t_cap, seq_lens=sl, tokens_per_split=split)
        got = cq.cq_decode_attention_paged(qd, kp, vp, ckd, cvd, 0.09, fmt, T, pages, seq_lens=sl, tokens_per_split=split)
        torch.cuda.synchronize()
        assert torch.equal(ref.view(torch.int16), got.view(torch.int16))
    # and against the oracle once
    kcodes, vcodes = cache_to_codes(kc, fmt, B, t_cap, T), cache_to_codes(vc, fmt, B, t_cap, T)
    got = cq.cq_decode_attention_paged(qd, kp, vp, ckd, cvd, 0.09, fmt, T, pages)
    check_attention(got.cpu().numpy(), O.attention(q, kcodes, vcodes, ck, cv, 0.09, hkv))


@pytest.mark.parametrize("c,b", [(8, 8), (2, 8), (8, 10)])
def test_paged_prefill_of_a_large_call_equals_the_contiguous_one(c, b):
    # enough (tile, head, sequence, tensor) items for the workgroup shapes that serve several tiles
    # (33 tiles per sequence: the last workgroup of a sequence has tiles to skip), appended at an
    # offset that leaves the first tile ragged
    hkv, hq, B, T, t_off = 32, 32, 2, 2100, 30
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(90 + c, 0, "k", D), synth.tensor_recipe(90 + c, 0, "v", D)
    xk = synth.sample_activations_torch(rk, B * T, 3, "cuda").reshape(B, T, D)
    xv = synth.sample_activations_torch(rv, B * T, 4, "cuda").reshape(B, T, D)
    ckd, cvd = dev(synth.sample_codebook(rk, c, b)), dev(synth.sample_codebook(rv, c, b))
    tiles = -(-(t_off + T) // 64)
    t_cap = tiles * 64
    n_pages = B * tiles + 7
    perm = np.random.default_rng(c).permutation(n_pages)
    table = perm[:B * tiles].reshape(B, tiles)
    pages = cq.PageTable(dev(table.astype(np.int32)), n_pages)
    kc = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), 0xA5, dtype=torch.uint8, device="cuda")
    vc = torch.full_like(kc, 0xA5)
    cq.cq_encode_kv(xk, xv, ckd, cvd, fmt, kc, vc, t_off, t_cap)
    kp = torch.full((cq.cq_paged_cache_bytes(fmt, n_pages),), 0xA5, dtype=torch.uint8, device="cuda")
    vp = torch.full_like(kp, 0xA5)
    cq.cq_encode_kv_paged(xk, xv, ckd, cvd, fmt, kp, vp, pages, t_off)
    torch.cuda.synchronize()
    assert torch.equal(_pool_to_cache(kp, fmt, table, n_pages), kc)
    assert torch.equal(_pool_to_cache(vp, fmt, table, n_pages), vc)
    # (the contiguous call at this size against the oracle, on sampled rows)
    from gpu_util import check_codes
    codes = cache_to_codes(kc, fmt, B, t_cap, T, t_off)
    rows = np.array([0, 33, 34, 1000, T - 65, T - 1])
    check_codes(codes[1, rows], xk[1, rows].cpu().numpy(), synth.sample_codebook(rk, c, b))


@pytest.mark.parametrize("c,b", FORMATS)
def test_paged_decode_step_equals_the_contiguous_step(c, b):
    hkv, hq, B, T = 2, 4, 3, 200
    fmt, xk, xv, ck, cv, q, tiles, n_pages, perm, pages = _setup(20 + c + b, c, b, hkv, hq, B, T)
    t_cap = tiles * 64
    table = perm[:B * tiles].reshape(B, tiles)
    ckd, cvd, qd = dev(ck), dev(cv), dev(q)
    kc = torch.zeros(cq.cq_cache_bytes(fmt, B, t_cap), dtype=torch.uint8, device="cuda")
    vc = torch.zeros_like(kc)
    kp = torch.zeros(cq.cq_paged_cache_bytes(fmt, n_pages), dtype=torch.uint8, device="cuda")
    vp = torch.zeros_like(kp)
    cq.cq_encode_kv(dev(xk[:, :T - 1]), dev(xv[:, :T - 1]), ckd, cvd, fmt, kc, vc, 0, t_cap)
    cq.cq_encode_kv_paged(dev(xk[:, :T - 1]), dev(xv[:, :T - 1]), ckd, cvd, fmt, kp, vp, pages, 0)
    lens = np.array([T, 65, 1], dtype=np.int32)
    for sl in (None, dev(lens)):
        k1, v1, k2, v2 = kc.clone(), vc.clone(), kp.clone(), vp.clone()
        xk1, xv1 = dev(xk[:, T - 1]), dev(xv[:, T - 1])
        ref = cq.cq_decode_step(qd, xk1, xv1, k1, v1, ckd, cvd, 0.1, fmt, T, t_cap, seq_lens=sl)
        got = cq.cq_decode_step_paged(qd, xk1, xv1, k2, v2, ckd, cvd, 0.1, fmt, T, pages, seq_lens=sl)
        torch.cuda.synchronize()
        assert torch.equal(ref.view(torch.int16), got.view(torch.int16))
        assert torch.equal(_pool_to_cache(k2, fmt, table, n_pages), k1)
        assert torch.equal(_pool_to_cache(v2, fmt, table, n_pages), v1)


def test_out_of_range_table_entries_are_clamped_not_followed():
    c, b, hkv, hq, B, T = 8, 8, 1, 1, 1, 64
    fmt = cq.CQFormat(c, b, 128, hkv)
    rk = synth.tensor_recipe(99, 0, "k", 128)
    ck = dev(synth.sample_codebook(rk, c, b))
    q = dev(np.ones((1, 1, 128), dtype=np.float16))
    pool = torch.zeros(cq.cq_paged_cache_bytes(fmt, 2), dtype=torch.uint8, device="cuda")
    for bad in (-5, 1000000):
        pages = cq.PageTable(dev(np.array([[bad]], dtype=np.int32)), 2)
        out = cq.cq_decode_attention_paged(q, pool, pool.clone(), ck, ck, 0.1, fmt, T, pages)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out.float()).all())
