"""The merge of context splits inside the split kernel (the last split of a (sequence, query head)
to finish merges them all, found with a per-row arrival counter): same results as the separate
merge kernel, on many streams at once, beyond the number of streams that get counters, beyond the
number of rows a counter set holds, and call after call (every call must leave the counters at
zero for the next)."""
import math

import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O

from gpu_util import check_attention, codes_to_cache, dev

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


@pytest.mark.parametrize("c,b", [(8, 8), (4, 8), (2, 8), (8, 10)])
def test_many_streams_at_once_and_call_after_call(c, b):
    # 20 streams (more than get counter sets: the rest run the merge kernel), each with its own
    # problem of 3 to 7 splits and ragged lengths, launched back to back, four rounds with new
    # queries each; yardsticks: the same call on a stream without counters (bit for bit), the oracle
    n_streams, scale = 20, 1.0 / math.sqrt(128)
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    probs = []
    for i in range(n_streams):
        t = 900 + 137 * i
        fmt, ck, cv, kc, vc, q = _case(2, c, b, 2, 4, 2, t, 100 + i)
        t_cap = (t + 63) // 64 * 64
        lens = np.array([t, max(1, t // 3)], dtype=np.int32)
        split = 64 * (2 + i % 4)
        d = dict(fmt=fmt, t=t, t_cap=t_cap, split=split, q=dev(q), ck=dev(ck), cv=dev(cv), kcache=codes_to_cache(kc, fmt, t_cap),
                 vcache=codes_to_cache(vc, fmt, t_cap), lens=dev(lens), kc=kc, vc=vc, ck_np=ck, cv_np=cv, lens_np=lens)
        d["out"] = torch.empty((2, 4, 128), dtype=torch.float16, device="cuda")
        d["ws"] = torch.full((cq.cq_decode_workspace_bytes(fmt, 2, 4, t, split),), 0xA5, dtype=torch.uint8, device="cuda")
        d["call"], _ = cq.prepare_decode_attention(d["q"], d["kcache"], d["vcache"], d["ck"], d["cv"], scale, fmt, t, t_cap,
                                                   seq_lens=d["lens"], tokens_per_split=split, out=d["out"], workspace=d["ws"])
        probs.append(d)
    torch.cuda.synchronize()
    for rnd in range(4):
        # new queries every round (a merge that read a stale partial of the round before would show)
        for i, d in enumerate(probs):
            if rnd:
                d["q"].copy_(dev(np.random.default_rng(1000 * rnd + i).standard_normal(tuple(d["q"].shape)).astype(np.float16)))
            d["out"].fill_(float("nan"))
        torch.cuda.synchronize()
        for s, d in zip(streams, probs):
            d["call"](s)
        torch.cuda.synchronize()
        got = [d["out"].clone() for d in probs]
        # the same calls on the last stream, which has no counters (merge kernel): bit for bit
        for d, g in zip(probs, got):
            d["out"].fill_(float("nan"))
            d["call"](streams[-1])
            streams[-1].synchronize()
            assert torch.equal(d["out"].view(torch.int16), g.view(torch.int16))
        for i in (rnd, 7 + rnd, 19 - rnd):
            d = probs[i]
            check_attention(got[i].cpu().numpy(), O.attention(d["q"].cpu().numpy(), d["kc"], d["vc"], d["ck_np"], d["cv_np"], scale, 2,
                                                              seq_lens=d["lens_np"]))


def test_more_rows_than_a_counter_set_holds():
    # 65 sequences x 128 query heads = 8320 rows of two splits: beyond the 8192 counters of a set,
    # so this launch is merged by the merge kernel; sampled rows against the oracle
    c, b, B, hq, hkv, t = 8, 8, 65, 128, 32, 128
    fmt, ck, cv, kc, vc, q = _case(5, c, b, B, hq, hkv, t, 7)
    scale = 0.1
    out = cq.cq_decode_attention(dev(q), codes_to_cache(kc, fmt, t), codes_to_cache(vc, fmt, t), dev(ck), dev(cv), scale, fmt, t, t,
                                 tokens_per_split=64)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for n in (0, 31, 64):
        ref = O.attention(q[n:n + 1], kc[n:n + 1], vc[n:n + 1], ck, cv, scale, hkv)
        check_attention(got[n:n + 1], ref)


def test_fused_step_and_layer_batched_step_with_splits():
    # the fused step with several splits, and the same step of three layers in one launch (their rows
    # share one counter set): equal to per-layer calls bit for bit, caches included
    c, b, B, hq, hkv, T, t_cap = 4, 8, 2, 4, 2, 3000, 3008
    fmt = cq.CQFormat(c, b, 128, hkv)
    scale, split = 0.09, 704
    layers, want, caches = [], [], []
    for layer in range(3):
        _, ck, cv, kc, vc, q = _case(2, c, b, B, hq, hkv, T, 40 + layer)
        xk = np.stack([synth.sample_activations(synth.tensor_recipe(2, layer, "k", fmt.channels), 1, chunk=n)[0] for n in range(B)])
        xv = np.stack([synth.sample_activations(synth.tensor_recipe(2, layer, "v", fmt.channels), 1, chunk=n)[0] for n in range(B)])
        io = dict(q=dev(q), x_k_new=dev(xk), x_v_new=dev(xv), k_codes=codes_to_cache(kc, fmt, t_cap),
                  v_codes=codes_to_cache(vc, fmt, t_cap), k_centroids=dev(ck), v_centroids=dev(cv),
                  out=torch.empty((B, hq, 128), dtype=torch.float16, device="cuda"))
        k2, v2 = io["k_codes"].clone(), io["v_codes"].clone()
        want.append(cq.cq_decode_step(io["q"], io["x_k_new"], io["x_v_new"], k2, v2, io["k_centroids"], io["v_centroids"], scale, fmt,
                                      T, t_cap, tokens_per_split=split))
        caches.append((k2, v2))
        layers.append(io)
    table = cq.LayerTable(layers, fmt, t_cap)
    cq.prepare_decode_step_layers(table, scale, T, tokens_per_split=split)()
    torch.cuda.synchronize()
    for io, w, (k2, v2) in zip(layers, want, caches):
        assert torch.equal(io["out"].view(torch.int16), w.view(torch.int16))
        assert torch.equal(io["k_codes"], k2) and torch.equal(io["v_codes"], v2)
