"""GPU parity of cq_chunk_attention (causal attention of the last m tokens over the coded cache,
on the matrix cores) against the CPU oracle, element by element: every format, chunk sizes
below, at and above the 32-row wavefront block and the 128-row workgroup block, grouped queries,
contexts around the tile size, split contexts, ragged lengths, paged pools."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O

from gpu_util import check_attention, codes_to_cache, dev, gpu_attention

pytestmark = pytest.mark.gpu

CHUNK_FORMATS = [(8, 8), (4, 8), (2, 8), (8, 10)]


def _case(seed, c, b, hq, hkv, B, m, T):
    rng = np.random.default_rng(2000 + seed)
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    ck = synth.sample_codebook(synth.tensor_recipe(80 + seed, 0, "k", D), c, b)
    cv = synth.sample_codebook(synth.tensor_recipe(80 + seed, 0, "v", D), c, b)
    kc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    vc = rng.integers(0, 1 << b, size=(B, T, fmt.groups)).astype(np.uint16)
    q = rng.standard_normal((B, m, hq, 128)).astype(np.float16)
    return fmt, q, kc, vc, ck, cv


def _gpu(q, kcache, vcache, ck, cv, scale, fmt, T, t_cap, seq_lens=None, split=0):
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    out = cq.cq_chunk_attention(dev(q), kcache, vcache, dev(ck), dev(cv), scale, fmt, T, t_cap, seq_lens=sl,
                                tokens_per_split=split)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _check(out, ref):
    B, m, hq, d = ref.shape
    check_attention(out.reshape(B * m, hq, d), ref.reshape(B * m, hq, d))


@pytest.mark.parametrize("c,b", CHUNK_FORMATS)
@pytest.mark.parametrize("m,T", [(1, 1), (1, 200), (5, 5), (5, 64), (31, 65), (32, 300), (33, 129), (100, 1000)])
def test_chunk_attention_matches_oracle(c, b, m, T):
    hq, hkv, B, t_cap = 4, 2, 2, 1024
    fmt, q, kc, vc, ck, cv = _case(m + T, c, b, hq, hkv, B, m, T)
    scale = 1.0 / math.sqrt(128)
    ref = O.chunk_attention(q, kc, vc, ck, cv, scale, hkv)
    # split 0: the library's choice (chunks of one or two tokens go token by token through the
    # single-token kernel); an explicit split always runs the chunk kernel
    for split in (0, t_cap):
        out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, scale, fmt, T, t_cap, split=split)
        _check(out, ref)


@pytest.mark.parametrize("c,b", CHUNK_FORMATS)
def test_chunk_attention_splits_ragged_lengths_and_many_rows(c, b):
    # 70 query tokens x 4 query heads per KV head = 280 rows per KV head: three 128-row blocks
    hq, hkv, B, m, T, t_cap = 8, 2, 3, 70, 1500, 1536
    fmt, q, kc, vc, ck, cv = _case(7, c, b, hq, hkv, B, m, T)
    lens = np.array([1500, 70, 777], dtype=np.int32)
    ref = O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv, seq_lens=lens)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    outs = []
    for split in (0, 64, 512, 1536):
        out = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, seq_lens=lens, split=split)
        _check(out, ref)
        outs.append(out.astype(np.float64))
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) <= 2e-3 * np.max(np.abs(outs[0]))


def test_chunk_of_one_token_agrees_with_decode_attention():
    c, b, hq, hkv, B, T, t_cap = 4, 8, 8, 4, 2, 900, 960
    fmt, q, kc, vc, ck, cv = _case(3, c, b, hq, hkv, B, 1, T)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    dec = gpu_attention(q[:, 0], kcache, vcache, ck, cv, 0.1, fmt, T, t_cap)
    ref = O.attention(q[:, 0], kc, vc, ck, cv, 0.1, hkv)
    # by default a chunk of one token IS a single-token attention; the chunk kernel (explicit split) agrees
    out = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap)
    assert np.array_equal(out[:, 0].view(np.uint16), dec.view(np.uint16))
    out = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, split=t_cap)
    check_attention(out[:, 0], ref)
    assert np.max(np.abs(out[:, 0].astype(np.float64) - dec.astype(np.float64))) <= 2e-3 * np.max(np.abs(ref))


@pytest.mark.parametrize("c,b,hq,hkv", [(4, 8, 4, 4), (8, 8, 8, 2), (8, 10, 4, 1), (2, 8, 2, 2)])
def test_short_chunk_equals_token_by_token_decode_attention(c, b, hq, hkv):
    # m = 2 with ragged lengths (one sequence as short as the chunk): query j of sequence n is the
    # single-token attention over max(len_n, m) - m + j + 1 tokens, bit for bit, and matches the oracle
    B, m, T, t_cap = 3, 2, 700, 704
    fmt, q, kc, vc, ck, cv = _case(11, c, b, hq, hkv, B, m, T)
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    lens = np.array([700, 2, 333], dtype=np.int32)
    out = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, seq_lens=lens)
    _check(out, O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv, seq_lens=lens))
    for j in range(m):
        lj = lens - (m - 1 - j)
        dec = gpu_attention(np.ascontiguousarray(q[:, j]), kcache, vcache, ck, cv, 0.1, fmt, T - (m - 1 - j), t_cap, seq_lens=lj)
        assert np.array_equal(out[:, j].view(np.uint16), dec.view(np.uint16))
    # the chunk kernel on the same inputs (explicit split) agrees within the tolerance
    alt = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, seq_lens=lens, split=256)
    assert np.max(np.abs(alt.astype(np.float64) - out.astype(np.float64))) <= 2e-3 * np.max(np.abs(out.astype(np.float64)))


@pytest.mark.parametrize("m", [8, 9])
def test_chunk_around_the_token_by_token_limit_of_a_large_batch(m):
    # 16 sequences x 32 KV heads x 32 tiles = 16384 tiles: a large batch, where chunks of up to
    # 8 tokens (one query head per KV head) go token by token and 9 tokens go to the matrix cores
    c, b, hq, hkv, B, T, t_cap = 8, 8, 32, 32, 16, 2048, 2048
    fmt, q, kc, vc, ck, cv = _case(13, c, b, hq, hkv, B, m, T)
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, 0.09, fmt, T, t_cap)
    # the oracle on three of the sixteen sequences
    pick = [0, 7, 15]
    ref = O.chunk_attention(q[pick], kc[pick], vc[pick], ck, cv, 0.09, hkv)
    _check(out[pick], ref)


def test_short_chunk_splits_long_contexts():
    # a context long enough for the token-by-token path to split it (and to need the workspace)
    c, b, hq, hkv, B, m, T, t_cap = 8, 8, 2, 2, 1, 2, 20000, 20032
    fmt, q, kc, vc, ck, cv = _case(12, c, b, hq, hkv, B, m, T)
    assert cq.cq_chunk_workspace_bytes(fmt, B, hq, m, T) > 0
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, 0.1, fmt, T, t_cap)
    _check(out, O.chunk_attention(q, kc, vc, ck, cv, 0.1, hkv))


def test_chunk_whole_sequence_first_query_returns_its_own_value():
    # m = T: query 0 sees token 0 only, so its output is that token's dequantized value (one fp16 rounding)
    c, b, hq, hkv, B, T, t_cap = 8, 8, 2, 2, 1, 150, 192
    fmt, q, kc, vc, ck, cv = _case(4, c, b, hq, hkv, B, T, T)
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, 0.2, fmt, T, t_cap)
    v0 = O.dequantize(vc[:, 0], cv).reshape(B, hkv, 128)
    assert np.max(np.abs(out[:, 0].astype(np.float64) - v0) / np.maximum(np.abs(v0), 1e-6)) <= 2.0 ** -10
    _check(out, O.chunk_attention(q, kc, vc, ck, cv, 0.2, hkv))


@pytest.mark.parametrize("m,split", [(40, 256), (2, 0)])       # the matrix-core kernel; the token-by-token path
def test_chunk_paged_equals_contiguous_bit_for_bit(m, split):
    c, b, hq, hkv, B, T, t_cap = 4, 8, 8, 4, 3, 900, 960
    fmt, q, kc, vc, ck, cv = _case(8, c, b, hq, hkv, B, m, T)
    n_tiles = t_cap // 64
    kcache, vcache = codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap)
    lens = np.array([900, 130, 64], dtype=np.int32)
    want = _gpu(q, kcache, vcache, ck, cv, 0.1, fmt, T, t_cap, seq_lens=lens, split=split)
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
    got = cq.cq_chunk_attention_paged(dev(q), pools[0], pools[1], dev(ck), dev(cv), 0.1, fmt, T, pages,
                                      seq_lens=dev(lens), tokens_per_split=split)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint16), want.view(np.uint16))


def test_chunk_rejects_short_sequences():
    fmt, q, kc, vc, ck, cv = _case(2, 8, 8, 2, 2, 1, 4, 64)
    with pytest.raises(cq.CQError):      # fewer cached tokens than queries
        cq.cq_chunk_attention(dev(q), codes_to_cache(kc, fmt, 64), codes_to_cache(vc, fmt, 64), dev(ck), dev(cv), 0.1, fmt, 3, 64)


def _sweep_cases():
    rng = np.random.default_rng(20240503)
    cases = []
    for i in range(16):
        c, b = CHUNK_FORMATS[i % 4]
        hkv = int(rng.choice([1, 2, 3, 8]))
        qper = int(rng.choice([1, 2, 4, 8]))
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 64, 127, 129, 500, 1337]))
        m = int(min(T, rng.choice([1, 2, 7, 33, 64, 150])))
        tiles = -(-T // 64)
        split_tiles = int(rng.integers(1, tiles + 1)) if rng.random() < 0.5 else 0
        ragged = bool(rng.random() < 0.5)
        cases.append((i, c, b, hkv * qper, hkv, B, m, T, split_tiles * 64, ragged))
    return cases


@pytest.mark.parametrize("case", _sweep_cases(), ids=lambda cs: "case%d-%dc%db-hq%d-hkv%d-B%d-m%d-T%d-split%d-%s" % (
    cs[:9] + ("ragged" if cs[9] else "full",)))
def test_chunk_attention_sweep(case):
    i, c, b, hq, hkv, B, m, T, split, ragged = case
    fmt, q, kc, vc, ck, cv = _case(100 + i, c, b, hq, hkv, B, m, T)
    t_cap = -(-T // 64) * 64
    lens = None
    if ragged:
        lens = np.random.default_rng(i).integers(m, T + 1, size=B).astype(np.int32)
    ref = O.chunk_attention(q, kc, vc, ck, cv, 0.09, hkv, seq_lens=lens)
    out = _gpu(q, codes_to_cache(kc, fmt, t_cap), codes_to_cache(vc, fmt, t_cap), ck, cv, 0.09, fmt, T, t_cap,
               seq_lens=lens, split=split)
    _check(out, ref)
