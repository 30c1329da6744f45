"""cq_decode_step_layers (several layers in one launch) against per-layer cq_decode_step calls:
outputs and caches bit for bit, every format, one and several splits, ragged lengths, the head
counts that take the XCD-aware workgroup numbering and those that do not."""
import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth

from gpu_util import dev

pytestmark = pytest.mark.gpu

FORMATS = [(8, 8), (4, 8), (2, 8), (8, 10)]


def _layers(seed, c, b, hq, hkv, B, T, t_cap, n_layers):
    """Per layer: codebooks, caches filled with T - 1 encoded tokens, the new rows, a query."""
    fmt = cq.CQFormat(c, b, 128, hkv)
    D = hkv * 128
    layers = []
    for l in range(n_layers):
        rk, rv = synth.tensor_recipe(seed, l, "k", D), synth.tensor_recipe(seed, l, "v", D)
        ck, cv = dev(synth.sample_codebook(rk, c, b)), dev(synth.sample_codebook(rv, c, b))
        kc = torch.full((cq.cq_cache_bytes(fmt, B, t_cap),), 0x3C, dtype=torch.uint8, device="cuda")
        vc = torch.full_like(kc, 0xC3)
        if T > 1:
            xk = np.stack([synth.sample_activations(rk, T - 1, chunk=10 * l + n) for n in range(B)])
            xv = np.stack([synth.sample_activations(rv, T - 1, chunk=10 * l + n) for n in range(B)])
            cq.cq_encode_kv(dev(xk), dev(xv), ck, cv, fmt, kc, vc, 0, t_cap)
        xk1 = np.concatenate([synth.sample_activations(rk, 1, chunk=500 + 10 * l + n) for n in range(B)])
        xv1 = np.concatenate([synth.sample_activations(rv, 1, chunk=500 + 10 * l + n) for n in range(B)])
        q = synth.sample_query(seed, l, B, hq, 128)
        layers.append(dict(q=dev(q), x_k_new=dev(xk1), x_v_new=dev(xv1), k_codes=kc, v_codes=vc,
                           k_centroids=ck, v_centroids=cv))
    torch.cuda.synchronize()
    return fmt, layers


def _compare(fmt, layers, T, t_cap, scale, seq_lens=None, split=0):
    sl = None if seq_lens is None else dev(np.asarray(seq_lens, dtype=np.int32))
    # reference: one cq_decode_step per layer on copies of the caches
    want = []
    for lay in layers:
        kc, vc = lay["k_codes"].clone(), lay["v_codes"].clone()
        out = cq.cq_decode_step(lay["q"], lay["x_k_new"], lay["x_v_new"], kc, vc, lay["k_centroids"], lay["v_centroids"],
                                scale, fmt, T, t_cap, seq_lens=sl, tokens_per_split=split)
        want.append((out, kc, vc))
    for lay in layers:
        lay["out"] = torch.full((lay["q"].shape[0], lay["q"].shape[1], 128), float("nan"), dtype=torch.float16, device="cuda")
    table = cq.LayerTable(layers, fmt, t_cap)
    outs = cq.cq_decode_step_layers(table, scale, T, seq_lens=sl, tokens_per_split=split)
    torch.cuda.synchronize()
    for l, (lay, (out, kc, vc)) in enumerate(zip(layers, want)):
        assert torch.equal(outs[l].view(torch.int16), out.view(torch.int16)), f"layer {l}: outputs differ"
        assert torch.equal(lay["k_codes"], kc) and torch.equal(lay["v_codes"], vc), f"layer {l}: caches differ"


@pytest.mark.parametrize("c,b", FORMATS)
@pytest.mark.parametrize("hq,hkv,T,split", [(4, 4, 300, 0), (8, 2, 1000, 256), (16, 8, 130, 64), (8, 8, 1, 0)])
def test_layered_step_equals_per_layer_steps(c, b, hq, hkv, T, split):
    t_cap = 1024
    fmt, layers = _layers(61, c, b, hq, hkv, 2, T, t_cap, 3)
    _compare(fmt, layers, T, t_cap, 0.09, split=split)


def test_layered_step_ragged_lengths_and_one_layer():
    c, b, hq, hkv, B, T, t_cap = 4, 8, 8, 4, 3, 700, 704
    fmt, layers = _layers(62, c, b, hq, hkv, B, T, t_cap, 2)
    _compare(fmt, layers, T, t_cap, 0.1, seq_lens=[700, 1, 65], split=128)
    fmt, layers = _layers(63, c, b, hq, hkv, B, T, t_cap, 1)
    _compare(fmt, layers, T, t_cap, 0.1)


def test_layer_table_refuses_shared_caches_and_bad_pointers():
    fmt, layers = _layers(64, 8, 8, 2, 2, 1, 10, 64, 2)
    for lay in layers:
        lay["out"] = torch.empty((1, 2, 128), dtype=torch.float16, device="cuda")
    bad = [dict(layers[0]), dict(layers[1])]
    bad[1]["k_codes"] = bad[0]["k_codes"]
    with pytest.raises(cq.CQError):
        cq.LayerTable(bad, fmt, 64)
    bad = [dict(layers[0]), dict(layers[1])]
    bad[1]["out"] = bad[0]["out"]
    with pytest.raises(cq.CQError):
        cq.LayerTable(bad, fmt, 64)
    bad = [dict(layers[0])]
    bad[0]["q"] = torch.empty(2 * 128 + 8, dtype=torch.float16, device="cuda")[4:4 + 256].view(1, 2, 128)   # 8-byte aligned only
    with pytest.raises(cq.CQError):
        cq.LayerTable(bad, fmt, 64)
    with pytest.raises(cq.CQError):          # workspace too small
        table = cq.LayerTable(layers, fmt, 64)
        cq.cq_decode_step_layers(table, 0.1, 10, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))


def test_layered_step_with_splits_beyond_8192_tokens():
    # CQ-8c8b with one 12288-token split per (sequence, head): the table form without replicas, layered
    c, b, hq, hkv, B, T, t_cap = 8, 8, 2, 1, 1, 12250, 12288
    fmt, layers = _layers(65, c, b, hq, hkv, B, T, t_cap, 2)
    _compare(fmt, layers, T, t_cap, 0.1, split=12288)
    fmt, layers = _layers(66, c, b, hq, hkv, B, T, t_cap, 2)
    _compare(fmt, layers, T, t_cap, 0.1, split=10944)
