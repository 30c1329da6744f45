"""The library under HIP graph capture: every entry point of the hot path only enqueues kernels on
the caller's stream (no allocation, no memset, no synchronisation), so a decode step captured
in a graph must replay to the eager result bit for bit — also on replays after the first, with
eager work and synchronisations between them."""
import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth

from gpu_util import dev

pytestmark = pytest.mark.gpu


def _setup(c, b, hq, hkv, B, T, t_cap, seed):
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    rk, rv = synth.tensor_recipe(seed, 0, "k", D), synth.tensor_recipe(seed, 0, "v", D)
    ck, cv = dev(synth.sample_codebook(rk, c, b)), dev(synth.sample_codebook(rv, c, b))
    kc = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), 0x11, dtype=torch.uint8, device="cuda")
    vc = torch.full_like(kc, 0x22)
    xk = np.stack([synth.sample_activations(rk, T - 1, chunk=n) for n in range(B)])
    xv = np.stack([synth.sample_activations(rv, T - 1, chunk=n) for n in range(B)])
    cq.cq_encode_kv(dev(xk), dev(xv), ck, cv, fmt, kc, vc, 0, t_cap)
    xk1 = dev(np.concatenate([synth.sample_activations(rk, 1, chunk=900 + n) for n in range(B)]))
    xv1 = dev(np.concatenate([synth.sample_activations(rv, 1, chunk=900 + n) for n in range(B)]))
    q = dev(synth.sample_query(seed, 0, B, hq, 128))
    torch.cuda.synchronize()
    return fmt, ck, cv, kc, vc, xk1, xv1, q


@pytest.mark.parametrize("c,b,hq,hkv,T,split", [(4, 8, 8, 8, 1000, 0), (8, 8, 8, 2, 3000, 1024), (8, 10, 4, 2, 700, 0),
                                                  (2, 8, 4, 4, 321, 128)])
def test_captured_decode_step_replays_to_the_eager_result(c, b, hq, hkv, T, split):
    B, t_cap = 3, 3072
    fmt, ck, cv, kc, vc, xk1, xv1, q = _setup(c, b, hq, hkv, B, T, t_cap, 60 + c + b)
    lens = dev(np.array([T, max(1, T // 3), T - 1], dtype=np.int32))
    scale = 0.1
    # eager reference on copies of the caches
    kc0, vc0 = kc.clone(), vc.clone()
    want_step = cq.cq_decode_step(q, xk1, xv1, kc0, vc0, ck, cv, scale, fmt, T, t_cap, seq_lens=lens, tokens_per_split=split)
    want_attn = cq.cq_decode_attention(q, kc0, vc0, ck, cv, scale, fmt, T, t_cap, seq_lens=lens, tokens_per_split=split)
    qc = torch.stack([q, q.flip(0)], dim=1).contiguous()                 # a chunk of two query tokens
    want_chunk = cq.cq_chunk_attention(qc, kc0, vc0, ck, cv, scale, fmt, T, t_cap)
    torch.cuda.synchronize()

    step, out_step = cq.prepare_decode_step(q, xk1, xv1, kc, vc, ck, cv, scale, fmt, T, t_cap, seq_lens=lens, tokens_per_split=split)
    attn, out_attn = cq.prepare_decode_attention(q, kc, vc, ck, cv, scale, fmt, T, t_cap, seq_lens=lens, tokens_per_split=split)
    chunk, out_chunk = cq.prepare_chunk_attention(qc, kc, vc, ck, cv, scale, fmt, T, t_cap)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side)
            attn(side)
            chunk(side)
    torch.cuda.synchronize()
    junk = torch.zeros(1 << 20, device="cuda")
    for replay in range(3):
        for o in (out_step, out_attn, out_chunk):
            o.fill_(float("nan"))
        junk.add_(1.0).sum().item()                                     # eager work and a synchronisation in between
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_step.view(torch.int16), want_step.view(torch.int16)), f"replay {replay}: step"
        assert torch.equal(out_attn.view(torch.int16), want_attn.view(torch.int16)), f"replay {replay}: attention"
        assert torch.equal(out_chunk.view(torch.int16), want_chunk.view(torch.int16)), f"replay {replay}: chunk"
        assert torch.equal(kc, kc0) and torch.equal(vc, vc0), f"replay {replay}: caches"
