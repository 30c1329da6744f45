"""cq_decode_attention_static (the entry point that allocates nothing: its context-split partials
live in the library's static scratch array) against cq_decode_attention with a caller's
workspace, through the C ABI: same kernels, so the outputs must be equal bit for bit -- on two
calls in a row, the second on a smaller input (which must not see what the first left in the
array), and both against the oracle."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O
import gpu_util as U

pytestmark = pytest.mark.gpu


def _case(cfg_id, c, b, batch, n_q, n_kv, t, seed):
    fmt = cq.CQFormat(c, b, 128, n_kv)
    rng = np.random.default_rng(seed)
    rk = synth.tensor_recipe(cfg_id, 0, "k", fmt.channels)
    rv = synth.tensor_recipe(cfg_id, 0, "v", fmt.channels)
    ck, cv = synth.sample_codebook(rk, c, b), synth.sample_codebook(rv, c, b)
    kc = rng.integers(0, 1 << b, size=(batch, t, fmt.groups)).astype(np.uint16)
    vc = rng.integers(0, 1 << b, size=(batch, t, fmt.groups)).astype(np.uint16)
    q = rng.standard_normal((batch, n_q, 128)).astype(np.float16)
    return fmt, ck, cv, kc, vc, q


def _run_both(fmt, ck, cv, kc, vc, q, t, split, seq_lens=None):
    t_cap = (t + 63) // 64 * 64
    kcache, vcache = U.codes_to_cache(kc, fmt, t_cap), U.codes_to_cache(vc, fmt, t_cap)
    scale = 1.0 / math.sqrt(128)
    dq, dck, dcv = U.dev(q), U.dev(ck), U.dev(cv)
    sl = None if seq_lens is None else U.dev(np.asarray(seq_lens, dtype=np.int32))
    ref_out = cq.cq_decode_attention(dq, kcache, vcache, dck, dcv, scale, fmt, t, t_cap, seq_lens=sl,
                                     tokens_per_split=split)
    out = torch.full_like(ref_out, float("nan"))
    call = cq.prepare_decode_attention_static(dq, kcache, vcache, dck, dcv, scale, fmt, t, t_cap, out,
                                              seq_lens=sl, tokens_per_split=split)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    call()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
    ref = O.attention(q, kc, vc, ck, cv, scale, fmt.n_kv_heads, seq_lens=seq_lens)
    U.check_attention(out.cpu().numpy(), ref)


def test_static_scratch_two_calls_second_smaller():
    # first call: 3 sequences x 8 query heads x 5 splits of 1024 tokens (ragged tail)
    fmt, ck, cv, kc, vc, q = _case(1, 8, 8, 3, 8, 8, 4200, 11)
    _run_both(fmt, ck, cv, kc, vc, q, 4200, 1024)
    # second call, smaller in every respect: fewer rows, fewer and shorter splits, ragged lengths
    fmt, ck, cv, kc, vc, q = _case(2, 4, 8, 2, 8, 8, 700, 12)
    _run_both(fmt, ck, cv, kc, vc, q, 700, 256, seq_lens=[700, 130])
    # and a call with a single split (uses none of the array)
    _run_both(fmt, ck, cv, kc, vc, q, 700, 0)


def test_static_scratch_grouped_queries_10_bit():
    fmt, ck, cv, kc, vc, q = _case(4, 8, 10, 2, 8, 2, 1500, 13)
    _run_both(fmt, ck, cv, kc, vc, q, 1500, 512)
    fmt, ck, cv, kc, vc, q = _case(4, 8, 10, 1, 4, 2, 300, 14)
    _run_both(fmt, ck, cv, kc, vc, q, 300, 128)


def test_static_scratch_rejects_what_does_not_fit():
    # 64 sequences x 32 heads x 8 splits x 520 B = 8.1 MiB of partials: more than the array holds
    fmt = cq.CQFormat(8, 8, 128, 32)
    t = 4096
    q = torch.zeros((64, 32, 128), dtype=torch.float16, device="cuda")
    cb = torch.zeros((fmt.groups, 256, 8), dtype=torch.float16, device="cuda")
    cache = torch.zeros(cq.cq_cache_bytes(fmt, 64, t), dtype=torch.uint8, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(cq.CQError) as e:
        cq.cq_decode_attention_static(q, cache, cache, cb, cb, 0.1, fmt, t, t, out, tokens_per_split=512)
    assert e.value.status == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    # the same problem with splits that fit is served
    cq.cq_decode_attention_static(q, cache, cache, cb, cb, 0.1, fmt, t, t, out, tokens_per_split=2048)
    torch.cuda.synchronize()
