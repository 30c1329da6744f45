"""GPU parity of decode attention over keys cached before the rotary position embedding
(cq_decode_attention_rope) against the CPU oracle (attention with rope_base), element by element:
every supported format, lengths around the tile size, split contexts, ragged batches, grouped
queries, paged pools, long contexts (large angles)."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O

from gpu_util import check_attention, codes_to_cache, dev, gpu_attention

pytestmark = pytest.mark.gpu

ROPE_FORMATS = [(8, 8), (4, 8), (2, 8)]
ATTN_FORMATS = ROPE_FORMATS + [(8, 10)]         # the 1024-centroid format reads its key centroids from L2
BASE = 10000.0


def _case(seed, c, b, hq, hkv, B, T):
    rng = np.random.default_rng(1000 + seed)
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    ck = synth.sample_codebook(synth.tensor_recipe(40 + seed, 0, "k", D), c, b)
    cv = synth.sample_codebook(synth.tensor_recipe(40 + seed, 0, "v", D), c, b)
    kc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    vc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    q = rng.standard_normal((B, hq, 128)).astype(np.float16)
    return fmt, q, kc, vc, ck, cv


def _gpu(q, kcache, vcache, ck, cv, scale, fmt, T, t_cap, rope, seq_lens=None, split=0):
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    out = cq.cq_decode_attention_rope(dev(q), kcache, vcache, dev(ck), dev(cv), scale, fmt, T, t_cap, rope,
                                      seq_lens=sl, tokens_per_split=split)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_rope_table_holds_cos_and_sin_of_tile_bases_and_lane_offsets():
    positions = 64 * 300
    rope = cq.RopeTable(BASE, positions)
    torch.cuda.synchronize()
    tab = rope.table.cpu().numpy().view(np.float32).reshape(-1, 2)
    theta = BASE ** (-2.0 * np.arange(64) / 128.0)
    tiles = (np.arange(300)[:, None] * 64.0) * theta[None, :]              # [tile][pair]
    lanes = theta[:, None] * np.arange(64.0)[None, :]                      # [pair][lane]
    want = np.concatenate([tiles.reshape(-1), lanes.reshape(-1)])
    assert tab.shape[0] == want.size
    # fp64 evaluation rounded once to fp32: half an ulp of a value <= 1, plus the fp64 error of the
    # angle (<= 2^-52 * 19200)
    assert np.max(np.abs(tab[:, 0] - np.cos(want))) <= 2.0 ** -24
    assert np.max(np.abs(tab[:, 1] - np.sin(want))) <= 2.0 ** -24


@pytest.mark.parametrize("c,b", ATTN_FORMATS)
@pytest.mark.parametrize("T", [1, 63, 64, 65, 1000])
def test_rope_attention_matches_oracle(c, b, T):
    hq, hkv, B, t_cap = 4, 2, 2, 1024
    fmt, q, kc, vc, ck, cv = _case(T, c, b, hq, hkv, B, T)
    scale = 1.0 / math.sqrt(128)
    rope = cq.RopeTable(BASE, 1024)
    ref = O.attention(q, kc, vc, ck, cv, scale, hkv, rope_base=BASE)
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, scale, fmt, T, t_cap, rope)
    check_attention(out, ref)
    # the rotation matters: without it the result is a different one (except for a single token,
    # where the output is the value row whatever the score)
    if T > 1:
        plain = O.attention(q, kc, vc, ck, cv, scale, hkv)
        assert np.max(np.abs(plain - ref)) > 1e-2 * np.max(np.abs(ref))


@pytest.mark.parametrize("c,b", ATTN_FORMATS)
def test_rope_split_invariance_and_ragged_lengths(c, b):
    hq, hkv, B, T, t_cap = 4, 4, 3, 5000, 5056
    fmt, q, kc, vc, ck, cv = _case(7, c, b, hq, hkv, B, T)
    scale = 0.11
    lens = np.array([5000, 1, 2500], dtype=np.int32)
    rope = cq.RopeTable(BASE, 8192)                    # longer than the cache: only a prefix is read
    ref = O.attention(q, kc, vc, ck, cv, scale, hkv, seq_lens=lens, rope_base=BASE)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    outs = []
    for split in (0, 64, 448, 4032, 8192):
        out = _gpu(q, kcache, vcache, ck, cv, scale, fmt, T, t_cap, rope, seq_lens=lens, split=split)
        check_attention(out, ref)
        outs.append(out.astype(np.float64))
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) <= 2e-3 * np.max(np.abs(outs[0]))


def test_rope_grouped_queries_and_eight_kv_heads():
    # 8 KV heads: the workgroup numbering that keeps a KV head on one XCD; 4 query heads per KV head
    c, b, hq, hkv, B, T, t_cap = 4, 8, 32, 8, 2, 700, 704
    fmt, q, kc, vc, ck, cv = _case(3, c, b, hq, hkv, B, T)
    rope = cq.RopeTable(BASE, t_cap)
    ref = O.attention(q, kc, vc, ck, cv, 0.09, hkv, rope_base=BASE)
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, 0.09, fmt, T, t_cap, rope)
    check_attention(out, ref)


@pytest.mark.parametrize("c,b", ROPE_FORMATS)
@pytest.mark.parametrize("hq,hkv", [(4, 2), (6, 2), (16, 2), (32, 8), (10, 1)])
def test_rope_grouped_queries_share_the_key_rotation(c, b, hq, hkv):
    # two or more query heads per KV head with byte codes: the kernel that rotates every key once
    # for (up to) four query heads.  2, 3, 8, 4 and 10 query heads per KV head (a partly filled
    # last group of four included), ragged lengths, one and several splits; at the split limit of
    # that kernel and one tile beyond it (where the per-head kernel takes over).
    B, T, t_cap = 2, 6100, 6144
    fmt, q, kc, vc, ck, cv = _case(11 + hq, c, b, hq, hkv, B, T)
    scale = 0.1
    lens = np.array([T, 2300], dtype=np.int32)
    rope = cq.RopeTable(BASE, t_cap)
    ref = O.attention(q, kc, vc, ck, cv, scale, hkv, seq_lens=lens, rope_base=BASE)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    for split in (0, 64 * 88, 64 * 89, 64 * 7):
        check_attention(_gpu(q, kcache, vcache, ck, cv, scale, fmt, T, t_cap, rope, seq_lens=lens, split=split), ref)
    assert cq.cq_decode_rope_default_split(fmt, B, hq, T) <= 64 * 88


def test_rope_long_context_and_other_base():
    # positions up to 40000: angles of tens of thousands of radians for the fast pairs
    c, b, hq, hkv, B, T = 8, 8, 2, 1, 1, 40000
    t_cap = 40000 // 64 * 64 + 64
    fmt, q, kc, vc, ck, cv = _case(5, c, b, hq, hkv, B, T)
    base = 500000.0
    rope = cq.RopeTable(base, t_cap)
    ref = O.attention(q, kc, vc, ck, cv, 0.1, hkv, rope_base=base)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    for split in (0, 16384):                # the library's split, and the longest one a workgroup takes
        check_attention(_gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, rope, split=split), ref)


def test_rope_zero_query_gives_the_uniform_weights_of_plain_attention():
    # q = 0: every score is 0 whatever the rotation, so the result equals the position-independent
    # kernel's bit for bit (same bins, same epilogue)
    c, b, hq, hkv, B, T, t_cap = 4, 8, 2, 2, 1, 300, 320
    fmt, q, kc, vc, ck, cv = _case(6, c, b, hq, hkv, B, T)
    rope = cq.RopeTable(BASE, t_cap)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    out0 = _gpu(np.zeros_like(q), kcache, vcache, ck, cv, 1.0, fmt, T, t_cap, rope)
    plain0 = gpu_attention(np.zeros_like(q), kcache, vcache, ck, cv, 1.0, fmt, T, t_cap)
    assert np.array_equal(out0.view(np.uint16), plain0.view(np.uint16))


def test_rope_paged_equals_contiguous_bit_for_bit():
    c, b, hq, hkv, B, T = 4, 8, 8, 4, 3, 900
    fmt, q, kc, vc, ck, cv = _case(8, c, b, hq, hkv, B, T)
    t_cap = 960
    n_tiles = t_cap // 64
    rope = cq.RopeTable(BASE, 1024)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    lens = np.array([900, 130, 64], dtype=np.int32)
    want = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, rope, seq_lens=lens, split=256)
    # scatter the tiles over a pool in a random page order
    rng = np.random.default_rng(9)
    n_pages = B * n_tiles + 5
    perm = rng.permutation(n_pages)[:B * n_tiles].astype(np.int32).reshape(B, n_tiles)
    tb = cq.cq_code_bytes_per_token_head(fmt) * 64
    pools = []
    for cache in (kcache, vcache):
        src = cache.cpu().numpy().reshape(B, hkv, n_tiles, tb)
        pool = np.full((n_pages, hkv, tb), 0x77, dtype=np.uint8)
        for n in range(B):
            for i in range(n_tiles):
                pool[perm[n, i]] = src[n, :, i]
        pools.append(dev(pool.reshape(-1)))
    pages = cq.PageTable(dev(perm), n_pages)
    got = cq.cq_decode_attention_rope_paged(dev(q), pools[0], pools[1], dev(ck), dev(cv), 0.1, fmt, T, pages, rope,
                                            seq_lens=dev(lens), tokens_per_split=256)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint16), want.view(np.uint16))


# ------------------------------------------------------------------------------------------
# fused decode step on pre-rotation caches
# ------------------------------------------------------------------------------------------
def _step_case(seed, c, b, hq, hkv, B, T, t_cap):
    """Caches holding T - 1 encoded tokens per sequence, the new (pre-rotation) rows, a query."""
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(70 + seed, 0, "k", D), synth.tensor_recipe(70 + seed, 0, "v", D)
    ck, cv = dev(synth.sample_codebook(rk, c, b)), dev(synth.sample_codebook(rv, c, b))
    kc = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), 0x3C, dtype=torch.uint8, device="cuda")
    vc = torch.full_like(kc, 0xC3)
    if T > 1:
        xk = np.stack([synth.sample_activations(rk, T - 1, chunk=n) for n in range(B)])
        xv = np.stack([synth.sample_activations(rv, T - 1, chunk=n) for n in range(B)])
        cq.cq_encode_kv(dev(xk), dev(xv), ck, cv, fmt, kc, vc, 0, t_cap)
    xk1 = np.concatenate([synth.sample_activations(rk, 1, chunk=500 + n) for n in range(B)])
    xv1 = np.concatenate([synth.sample_activations(rv, 1, chunk=500 + n) for n in range(B)])
    q = dev(synth.sample_query(70 + seed, 0, B, hq, 128))
    torch.cuda.synchronize()
    return fmt, q, dev(xk1), dev(xv1), kc, vc, ck, cv


@pytest.mark.parametrize("c,b", ATTN_FORMATS)
@pytest.mark.parametrize("hq,hkv,T,split", [(4, 4, 1, 0), (4, 4, 64, 0), (8, 2, 65, 0), (4, 2, 1000, 0),
                                            (4, 4, 1000, 256), (16, 8, 300, 64)])
def test_rope_step_equals_encode_then_rope_attention(c, b, hq, hkv, T, split):
    B, t_cap = 2, 1024
    fmt, q, xk1, xv1, kc, vc, ck, cv = _step_case(T, c, b, hq, hkv, B, T, t_cap)
    rope = cq.RopeTable(BASE, t_cap)
    kc2, vc2 = kc.clone(), vc.clone()
    cq.cq_encode_kv(xk1.view(B, 1, -1), xv1.view(B, 1, -1), ck, cv, fmt, kc2, vc2, T - 1, t_cap)
    want = cq.cq_decode_attention_rope(q, kc2, vc2, ck, cv, 0.09, fmt, T, t_cap, rope, tokens_per_split=split)
    got = cq.cq_decode_step_rope(q, xk1, xv1, kc, vc, ck, cv, 0.09, fmt, T, t_cap, rope, tokens_per_split=split)
    torch.cuda.synchronize()
    assert torch.equal(kc, kc2) and torch.equal(vc, vc2), "stored codes differ from cq_encode_kv"
    assert torch.equal(got.view(torch.int16), want.view(torch.int16)), "outputs differ"


@pytest.mark.parametrize("c,b", [(4, 8), (8, 10)])
def test_rope_step_ragged_lengths_and_oracle(c, b):
    # sequences of different lengths: each new token lands at its own position; also against the
    # oracle end to end (codes of the new rows, then attention with rotation)
    hq, hkv, B, T, t_cap = 8, 4, 3, 700, 704
    fmt, q, xk1, xv1, kc, vc, ck, cv = _step_case(9, c, b, hq, hkv, B, T, t_cap)
    rope = cq.RopeTable(BASE, t_cap)
    lens = np.array([700, 1, 65], dtype=np.int32)
    kc2, vc2 = kc.clone(), vc.clone()
    per_seq = kc.numel() // B
    for n in range(B):
        sl = slice(n * per_seq, (n + 1) * per_seq)
        cq.cq_encode_kv(xk1[n].view(1, 1, -1), xv1[n].view(1, 1, -1), ck, cv, fmt, kc2[sl], vc2[sl], int(lens[n]) - 1, t_cap)
    want = cq.cq_decode_attention_rope(q, kc2, vc2, ck, cv, 0.1, fmt, T, t_cap, rope, seq_lens=dev(lens), tokens_per_split=128)
    got = cq.cq_decode_step_rope(q, xk1, xv1, kc, vc, ck, cv, 0.1, fmt, T, t_cap, rope, seq_lens=dev(lens), tokens_per_split=128)
    torch.cuda.synchronize()
    assert torch.equal(kc, kc2) and torch.equal(vc, vc2)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    from gpu_util import cache_to_codes
    kcodes, vcodes = cache_to_codes(kc, fmt, B, t_cap, T), cache_to_codes(vc, fmt, B, t_cap, T)
    ref = O.attention(q.cpu().numpy(), kcodes, vcodes, ck.cpu().numpy(), cv.cpu().numpy(), 0.1, hkv, seq_lens=lens,
                      rope_base=BASE)
    check_attention(got.cpu().numpy(), ref)
    for n in range(B):
        p = int(lens[n]) - 1
        for codes, x1, cb in ((kcodes, xk1, ck), (vcodes, xv1, cv)):
            wantc, d1, d2 = O.encode(x1[n:n + 1].cpu().numpy(), cb.cpu().numpy(), with_distances=True)
            assert not ((codes[n, p:p + 1] != wantc) & ~((d2 - d1) < 1e-6 * d2)).any()


@pytest.mark.parametrize("c,b", [(8, 8), (8, 10)])
def test_rope_step_paged_equals_contiguous(c, b):
    hq, hkv, B, T, t_cap = 4, 4, 2, 200, 256
    fmt, q, xk1, xv1, kc, vc, ck, cv = _step_case(10, c, b, hq, hkv, B, T, t_cap)
    rope = cq.RopeTable(BASE, t_cap)
    n_tiles = t_cap // 64
    n_pages = B * n_tiles + 3
    rng = np.random.default_rng(3)
    perm = rng.permutation(n_pages)[:B * n_tiles].astype(np.int32).reshape(B, n_tiles)
    tb = cq.cq_code_bytes_per_token_head(fmt) * 64
    pools = []
    for cache in (kc, vc):
        src = cache.cpu().numpy().reshape(B, hkv, n_tiles, tb)
        pool = np.full((n_pages, hkv, tb), 0x77, dtype=np.uint8)
        for n in range(B):
            for i in range(n_tiles):
                pool[perm[n, i]] = src[n, :, i]
        pools.append(dev(pool.reshape(-1)))
    pages = cq.PageTable(dev(perm), n_pages)
    want = cq.cq_decode_step_rope(q, xk1, xv1, kc, vc, ck, cv, 0.1, fmt, T, t_cap, rope)
    got = cq.cq_decode_step_rope_paged(q, xk1, xv1, pools[0], pools[1], ck, cv, 0.1, fmt, T, pages, rope)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    for cache, pool in ((kc, pools[0]), (vc, pools[1])):
        src = cache.cpu().numpy().reshape(B, hkv, n_tiles, tb)
        pl = pool.cpu().numpy().reshape(n_pages, hkv, tb)
        for n in range(B):
            for i in range(n_tiles):
                assert np.array_equal(pl[perm[n, i]], src[n, :, i])


def _rope_sweep_cases():
    rng = np.random.default_rng(24050391)
    cases = []
    for i in range(12):
        c, b = ROPE_FORMATS[i % 3]
        hkv = int(rng.choice([1, 2, 3, 8]))
        qper = int(rng.choice([1, 2, 4]))
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 64, 127, 129, 500, 1337, 2049]))
        tiles = -(-T // 64)
        split_tiles = int(rng.integers(1, min(tiles, 128) + 1)) if rng.random() < 0.6 else 0
        ragged = bool(rng.random() < 0.5)
        step = bool(rng.random() < 0.5)
        cases.append((i, c, b, hkv * qper, hkv, B, T, split_tiles * 64, ragged, step))
    return cases


@pytest.mark.parametrize("case", _rope_sweep_cases(), ids=lambda cs: "case%d-%dc%db-hq%d-hkv%d-B%d-T%d-split%d-%s-%s" % (
    cs[:8] + ("ragged" if cs[8] else "full", "step" if cs[9] else "attn")))
def test_rope_attention_and_step_sweep(case):
    i, c, b, hq, hkv, B, T, split, ragged, step = case
    fmt, q, kc, vc, ck, cv = _case(200 + i, c, b, hq, hkv, B, T)
    t_cap = -(-T // 64) * 64
    rope = cq.RopeTable(BASE, t_cap)
    lens = np.random.default_rng(i).integers(1, T + 1, size=B).astype(np.int32) if ragged else None
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    if step:
        # the newest token of every sequence comes in as fp16 rows instead of cached codes
        D = hkv * 128
        xk1 = np.concatenate([synth.sample_activations(synth.tensor_recipe(300 + i, 0, "k", D), 1, chunk=n) for n in range(B)])
        xv1 = np.concatenate([synth.sample_activations(synth.tensor_recipe(300 + i, 0, "v", D), 1, chunk=n) for n in range(B)])
        sl = None if lens is None else dev(lens)
        out = cq.cq_decode_step_rope(dev(q), dev(xk1), dev(xv1), kcache, vcache, dev(ck), dev(cv), 0.09, fmt, T, t_cap, rope,
                                     seq_lens=sl, tokens_per_split=split)
        torch.cuda.synchronize()
        from gpu_util import cache_to_codes
        kc, vc = cache_to_codes(kcache, fmt, B, t_cap, T), cache_to_codes(vcache, fmt, B, t_cap, T)
        out = out.cpu().numpy()
        for n in range(B):
            p = (T if lens is None else int(lens[n])) - 1
            for codes, x1, cb in ((kc, xk1, ck), (vc, xv1, cv)):
                want, d1, d2 = O.encode(x1[n:n + 1], cb, with_distances=True)
                assert not ((codes[n, p:p + 1] != want) & ~((d2 - d1) < 1e-6 * d2)).any()
    else:
        out = _gpu(q, kcache, vcache, ck, cv, 0.09, fmt, T, t_cap, rope, seq_lens=lens, split=split)
    ref = O.attention(q, kc, vc, ck, cv, 0.09, hkv, seq_lens=lens, rope_base=BASE)
    check_attention(out, ref)


# ------------------------------------------------------------------------------------------
# several query tokens over pre-rotation caches: the matrix-core kernel (key tiles rotated once
# per tile and KV head); chunks of one or two tokens token by token through the decode kernel
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("c,b", ATTN_FORMATS)
@pytest.mark.parametrize("hq,hkv,m,T,split", [(4, 4, 1, 1, 0), (4, 2, 2, 333, 0), (4, 2, 3, 3, 0), (8, 2, 5, 700, 0), (4, 4, 4, 1000, 256),
                                              (4, 2, 31, 65, 0), (4, 2, 33, 129, 1024), (4, 2, 100, 1000, 0)])
def test_rope_chunk_matches_oracle_and_token_by_token_calls(c, b, hq, hkv, m, T, split):
    B, t_cap = 3, 1024
    fmt, _, kc, vc, ck, cv = _case(50 + m + T, c, b, hq, hkv, B, T)
    q = np.random.default_rng(m * 1000 + T).standard_normal((B, m, hq, 128)).astype(np.float16)
    lens = np.array([T, max(m, T // 3), max(m, T - 1)], dtype=np.int32)
    rope = cq.RopeTable(BASE, t_cap)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    out = cq.cq_chunk_attention_rope(dev(q), kcache, vcache, dev(ck), dev(cv), 0.1, fmt, T, t_cap, rope,
                                     seq_lens=dev(lens), tokens_per_split=split)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    ref = O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv, seq_lens=lens, rope_base=BASE)
    check_attention(out.reshape(B * m, hq, 128), ref.reshape(B * m, hq, 128))
    for j in range(m if m <= 5 else 0):
        dec = _gpu(np.ascontiguousarray(q[:, j]), kcache, vcache, ck, cv, 0.1, fmt, T - (m - 1 - j), t_cap, rope,
                   seq_lens=lens - (m - 1 - j))
        if m <= 2 and split == 0:       # served token by token: the decode kernel's own results
            assert np.array_equal(out[:, j].view(np.uint16), dec.view(np.uint16))
        else:                           # the matrix-core kernel agrees with it within the tolerance
            assert np.max(np.abs(out[:, j].astype(np.float64) - dec.astype(np.float64))) <= 2e-3 * np.max(np.abs(ref[:, j]))


@pytest.mark.parametrize("c,b", ATTN_FORMATS)
def test_rope_chunk_splits_ragged_lengths_many_rows_and_far_positions(c, b):
    # 70 query tokens x 4 query heads per KV head = 280 rows per KV head (three 128-row blocks), context
    # splits, ragged lengths; then the same chunk at positions beyond 30000 (base 500000)
    hq, hkv, B, m, T, t_cap = 8, 2, 3, 70, 1500, 1536
    fmt, _, kc, vc, ck, cv = _case(7, c, b, hq, hkv, B, T)
    q = np.random.default_rng(70).standard_normal((B, m, hq, 128)).astype(np.float16)
    lens = np.array([1500, 70, 777], dtype=np.int32)
    ref = O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv, seq_lens=lens, rope_base=BASE)
    rope = cq.RopeTable(BASE, t_cap)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    for split in (0, 64, 512, 1536):
        out = cq.cq_chunk_attention_rope(dev(q), kcache, vcache, dev(ck), dev(cv), 0.1, fmt, T, t_cap, rope,
                                         seq_lens=dev(lens), tokens_per_split=split)
        torch.cuda.synchronize()
        check_attention(out.cpu().numpy().reshape(B * m, hq, 128), ref.reshape(B * m, hq, 128))
    hq, hkv, B, m, T, t_cap = 4, 1, 1, 40, 32000, 32000
    fmt, _, kc, vc, ck, cv = _case(8, c, b, hq, hkv, B, T)
    q = np.random.default_rng(71).standard_normal((B, m, hq, 128)).astype(np.float16)
    ref = O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv, rope_base=500000.0)
    out = cq.cq_chunk_attention_rope(dev(q), codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), dev(ck), dev(cv), 0.1, fmt,
                                     T, t_cap, cq.RopeTable(500000.0, t_cap))
    torch.cuda.synchronize()
    check_attention(out.cpu().numpy().reshape(B * m, hq, 128), ref.reshape(B * m, hq, 128))


def test_rope_chunk_paged_equals_contiguous():
    c, b, hq, hkv, B, m, T, t_cap = 4, 8, 8, 4, 2, 3, 500, 512
    fmt, _, kc, vc, ck, cv = _case(77, c, b, hq, hkv, B, T)
    q = np.random.default_rng(78).standard_normal((B, m, hq, 128)).astype(np.float16)
    rope = cq.RopeTable(BASE, t_cap)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    lens = dev(np.array([500, 77], dtype=np.int32))
    want = cq.cq_chunk_attention_rope(dev(q), kcache, vcache, dev(ck), dev(cv), 0.1, fmt, T, t_cap, rope, seq_lens=lens)
    n_tiles = t_cap // 64
    n_pages = B * n_tiles + 2
    perm = np.random.default_rng(5).permutation(n_pages)[:B * n_tiles].astype(np.int32).reshape(B, n_tiles)
    tb = cq.cq_code_bytes_per_token_head(fmt) * 64
    pools = []
    for cache in (kcache, vcache):
        src = cache.cpu().numpy().reshape(B, hkv, n_tiles, tb)
        pool = np.full((n_pages, hkv, tb), 0x77, dtype=np.uint8)
        for n in range(B):
            for i in range(n_tiles):
                pool[perm[n, i]] = src[n, :, i]
        pools.append(dev(pool.reshape(-1)))
    pages = cq.PageTable(dev(perm), n_pages)
    got = cq.cq_chunk_attention_rope_paged(dev(q), pools[0], pools[1], dev(ck), dev(cv), 0.1, fmt, T, pages, rope, seq_lens=lens)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
