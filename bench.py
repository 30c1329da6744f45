#!/usr/bin/env python3
"""Throughput of the CQ hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

Workload (the second named configuration): CQ-4c8b (2 bits per channel) on a Llama-2-7B-shaped
KV cache -- 32 layers, batch 16, 32 heads x 128, context 4096, MHA.  One STEP is one decode step
of the whole hot path over all 32 layers: per layer, encode the 16 new key rows and the 16 new
value rows into cache position 4095 and attend over all 4096 cached tokens -- one fused
cq_decode_step launch, bit-identical to cq_encode_kv followed by cq_decode_attention.  Every layer
has its own codebooks, caches, queries and new rows (4 GiB of codes in total, far more than the
256 MB last-level cache, so code reads are real HBM reads).

Inputs are synthetic and resident in HBM before the timed region: correlated-Gaussian K/V rows
(synth/generator.py) drawn on the device and REALLY encoded with cq_encode to fill the caches.

The timed region is K steps of 32 prepared calls in stream order, between two HIP events on the
launching stream and a host clock on both sides of a synchronize (the headline).  The same K
steps are also timed as replays of a captured HIP graph (reported beside it).

`extra` holds the other four named configurations and the remaining entry points, each decode
and encode entry with a `roofline` object of its own.  Every decode entry rotates over enough
independent cache sets that consecutive launches touch more than the 256 MB last-level cache
(`buffer_sets`, `cache_resident: false`).

One JSON line is printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published peak, GB/s
LAST_LEVEL_CACHE_BYTES = 256e6
# vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (the published
# 157.3 TFLOP/s of fp32 counts a packed FMA, 4 flops, per lane-instruction)
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
MFMA_SCORE_OPS = 1.25
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP16_MFMA_PEAK_TFLOPS = 2500.0
METRIC = "decode-attn KV tokens/s & achieved HBM GB/s (% peak); cq_encode tokens/s"
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(kernel_key: str):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_per_launch.txt: `key <tab> bytes <tab> provenance`), or None when the
    file has no line for it."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("#") or not line.strip():
                    continue
                parts = line.rstrip("\n").split("\t")
                if len(parts) >= 2 and parts[0] == kernel_key:
                    return float(parts[1])
    except OSError:
        pass
    return None


def hbm_roofline(kernel: str, traffic_key: str, code_bytes: int, ms: float, launches: int, **more):
    achieved = code_bytes / (ms * 1e-3) / 1e9
    r = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
         "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(traffic_key),
         "algorithmic_bytes_per_launch": code_bytes, "avg_launch_ms": ms, "launches_timed": launches}
    r.update(more)
    return r


def encode_roofline(kernel: str, tokens: int, channels: int, n_centroids: int, ms: float, mfma: bool):
    """cq_encode: D * 2^b (token channel, centroid) pairs per token.  The MFMA-filtered kernel spends
    1.25 vector lane-instructions per (token, centroid) score (c channels each) on finding the two
    largest (17 per 16 scores for the quad maxima and their running best and runner-up, the rest
    for the second look at the winning quad), the matrix cores do the multiply-adds; the direct
    kernel spends 2c + 3 per score.  MFMA_SCORE_OPS is that figure."""
    pairs = tokens * channels * n_centroids
    t = ms * 1e-3
    r = {"bound": "alu", "kernel": kernel, "unit": "T lane-instr/s", "peak": VALU_PEAK_LANE_OPS / 1e12,
         "algorithmic_flops_per_token": 3 * channels * n_centroids,
         "algorithmic_TFLOPs": 3 * pairs / t / 1e12, "fp32_vector_peak_TFLOPs": FP32_VECTOR_PEAK_TFLOPS,
         "avg_launch_ms": ms}
    return r, pairs / t


class LayerState:
    """Device buffers of one layer."""
    __slots__ = ("ck", "cv", "kcache", "vcache", "q", "xk_new", "xv_new", "out", "ws", "enc_kv", "dec", "step")


def build_workload(cq, synth, torch, cfg, n_layers, fill_chunk_tokens=16384):
    """Allocate and fill every layer's buffers.  Cache positions 0 .. T-2 come from encoding
    device-generated activations; the last position is written by the timed step itself."""
    import numpy as np
    fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
    B, T, D = cfg.batch, cfg.context, cfg.kv_channels
    t_cap = (T + 63) // 64 * 64
    layers = []
    dev = lambda a: torch.from_numpy(a).cuda()
    for layer in range(n_layers):
        st = LayerState()
        rk = synth.tensor_recipe(cfg.cfg_id, layer, "k", D)
        rv = synth.tensor_recipe(cfg.cfg_id, layer, "v", D)
        st.ck = dev(synth.sample_codebook(rk, cfg.c, cfg.b))
        st.cv = dev(synth.sample_codebook(rv, cfg.c, cfg.b))
        st.kcache = cq.alloc_cache(fmt, B, t_cap)
        st.vcache = cq.alloc_cache(fmt, B, t_cap)
        st.kcache.zero_()
        st.vcache.zero_()
        n_fill = T - cfg.encode_tokens if cfg.encode_tokens < T else T
        for recipe, cb, cache, sid in ((rk, st.ck, st.kcache, 0), (rv, st.cv, st.vcache, 1)):
            for n in range(B):
                t0 = 0
                while t0 < n_fill:
                    tn = min(fill_chunk_tokens, n_fill - t0)
                    x = synth.sample_activations_torch(recipe, tn, 7919 * n + 2 * t0 + sid, "cuda")
                    # one sequence at a time: view the cache of sequence n as a batch of 1
                    per_seq = cache.numel() // B
                    cq.cq_encode(x.view(1, tn, D), cb, fmt, cache[n * per_seq:(n + 1) * per_seq], t0, t_cap)
                    t0 += tn
                    del x
        st.q = dev(synth.sample_query(cfg.cfg_id, layer, B, cfg.n_q_heads, cfg.head_dim))
        tnew = min(cfg.encode_tokens, T)
        st.xk_new = dev(np.stack([synth.sample_activations(rk, tnew, chunk=1000 + n) for n in range(B)]))
        st.xv_new = dev(np.stack([synth.sample_activations(rv, tnew, chunk=1000 + n) for n in range(B)]))
        st.out = torch.empty((B, cfg.n_q_heads, cfg.head_dim), dtype=torch.float16, device="cuda")
        nws = cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, 0)
        st.ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
        layers.append(st)
        if layer % 8 == 7 or layer == n_layers - 1:
            torch.cuda.synchronize()
            log(f"[bench] layer {layer + 1}/{n_layers} caches filled")
    return fmt, t_cap, layers


def prepare_calls(cq, fmt, cfg, t_cap, layers, scale):
    """Marshal the three calls of every layer once; the step then only crosses the C ABI."""
    T = cfg.context
    t_off = T - layers[0].xk_new.shape[1]
    for st in layers:
        st.enc_kv = cq.prepare_encode_kv(st.xk_new, st.xv_new, st.ck, st.cv, fmt, st.kcache, st.vcache, t_off, t_cap)
        st.dec, _ = cq.prepare_decode_attention(st.q, st.kcache, st.vcache, st.ck, st.cv, scale, fmt, T, t_cap,
                                                out=st.out, workspace=st.ws)
        st.step, _ = cq.prepare_decode_step(st.q, st.xk_new[:, 0, :], st.xv_new[:, 0, :], st.kcache, st.vcache,
                                            st.ck, st.cv, scale, fmt, T, t_cap, out=st.out, workspace=st.ws)


def run_step(layers):
    """One decode step: per layer ONE cq_decode_step launch (encode the new K/V rows of the 16
    sequences into position T-1, then attend over all T positions)."""
    for st in layers:
        st.step()


def run_step_unfused(layers):
    """The same step as two launches per layer (cq_encode_kv, cq_decode_attention)."""
    for st in layers:
        st.enc_kv()
        st.dec()


def time_calls(torch, fn, iters, warmup=2):
    """Median and mean of `iters` calls of fn, each between its own HIP event pair."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], sum(ts) / len(ts)


def time_rotating(torch, calls, rounds, warmup=1):
    """Mean duration (ms) of one call when the calls (one per buffer set) are launched round robin,
    back to back, `rounds` times between ONE HIP event pair: launch-to-launch time, gaps included."""
    for _ in range(warmup):
        for c in calls:
            c()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(rounds):
        for c in calls:
            c()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (rounds * len(calls))


def sets_beyond_cache(code_bytes):
    """Buffer sets to rotate over so that a launch never finds its codes in the last-level cache:
    the sets touched between two uses of one set must exceed the cache."""
    return max(3, int(math.ceil(2.0 * LAST_LEVEL_CACHE_BYTES / code_bytes)) + 1)


def fill_cache_set(cq, synth, torch, cfg, fmt, set_id, chunk_tokens):
    """One set of device buffers of a configuration: codebooks (their own per set), K / V caches
    filled by really encoding generated activations, queries, output, workspace."""
    B, T, D = cfg.batch, cfg.context, cfg.kv_channels
    rk = synth.tensor_recipe(cfg.cfg_id, set_id, "k", D)
    rv = synth.tensor_recipe(cfg.cfg_id, set_id, "v", D)
    ck = torch.from_numpy(synth.sample_codebook(rk, cfg.c, cfg.b)).cuda()
    cv = torch.from_numpy(synth.sample_codebook(rv, cfg.c, cfg.b)).cuda()
    kcache, vcache = cq.alloc_cache(fmt, B, T), cq.alloc_cache(fmt, B, T)
    per_seq = kcache.numel() // B
    for n in range(B):
        for t0 in range(0, T, chunk_tokens):
            tn = min(chunk_tokens, T - t0)
            xk = synth.sample_activations_torch(rk, tn, 31 * n + t0, "cuda").view(1, tn, D)
            xv = synth.sample_activations_torch(rv, tn, 31 * n + t0 + 1, "cuda").view(1, tn, D)
            cq.cq_encode_kv(xk, xv, ck, cv, fmt, kcache[n * per_seq:(n + 1) * per_seq], vcache[n * per_seq:(n + 1) * per_seq], t0, T)
            del xk, xv
    q = torch.from_numpy(synth.sample_query(cfg.cfg_id, set_id, B, cfg.n_q_heads, cfg.head_dim)).cuda()
    out = torch.empty((B, cfg.n_q_heads, cfg.head_dim), dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, 0)), dtype=torch.uint8, device="cuda")
    return dict(ck=ck, cv=cv, kcache=kcache, vcache=vcache, q=q, out=out, ws=ws, rk=rk, rv=rv)


def kernel_name(cfg, step=False, ns=None):
    gh = cfg.head_dim // cfg.c
    if ns is None:
        tiles = (cfg.context + 63) // 64
        import paper_2405_03917_amd as cq
        fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
        split = cq.cq_decode_default_split(fmt, cfg.batch, cfg.n_q_heads, cfg.context) // 64
        per_wave = (min(split, tiles) + 7) // 8
        full = 32 if cfg.b == 10 else 16
        ns = full // 2 if per_wave <= full // 2 else full
    return f"decode_split_kernel<{gh}, {cfg.c}, {cfg.b}, {ns}, {'true' if step else 'false'}, false>"


def decode_config_entry(cq, synth, torch, cfg_id, rounds, label):
    """cq_decode_attention of one layer of a named configuration, rotating over cache sets."""
    cfg = synth.CONFIGS[cfg_id]
    fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
    B, T, D = cfg.batch, cfg.context, cfg.kv_channels
    code_bytes = B * T * 2 * D * cfg.b // (8 * cfg.c)
    n_sets = sets_beyond_cache(code_bytes)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    sets, calls = [], []
    for s in range(n_sets):
        st = fill_cache_set(cq, synth, torch, cfg, fmt, s, min(T, 32768))
        call, _ = cq.prepare_decode_attention(st["q"], st["kcache"], st["vcache"], st["ck"], st["cv"], scale, fmt, T, T,
                                              out=st["out"], workspace=st["ws"])
        sets.append(st)
        calls.append(call)
    torch.cuda.synchronize()
    ms = time_rotating(torch, calls, rounds)
    split = cq.cq_decode_default_split(fmt, B, cfg.n_q_heads, T)
    kname = kernel_name(cfg)
    entry = {"workload": f"{label}: cq_decode_attention of one layer, {cfg.n_q_heads} query / {cfg.n_kv_heads} KV heads, "
                         f"batch {B}, context {T}",
             "ms": ms, "kv_tokens_per_s": B * T / (ms * 1e-3), "code_read_GBps": code_bytes / (ms * 1e-3) / 1e9,
             "frac_of_hbm_peak": code_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "tokens_per_split": split,
             "splits_merged_in_kernel": split < T, "buffer_sets": n_sets, "cache_resident": False,
             "bytes_between_reuse": code_bytes * (n_sets - 1),
             "roofline": hbm_roofline(kname, kname, code_bytes, ms, rounds * n_sets)}
    return cfg, fmt, sets, entry


def extra_measurements(cq, synth, torch):
    """The other named configurations and entry points."""
    import numpy as np
    out = {}
    scale = 1.0 / math.sqrt(128)

    # ---- configuration 1: CQ-8c8b, batch 1, context 1024: encode all 1024 tokens of K and V, then one
    # decode step.  Latency-bound (1 MiB of codes); 64 buffer sets of 9 MiB (codebooks included).
    cfg = synth.CONFIGS[1]
    fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
    T, D = cfg.context, cfg.kv_channels
    n_sets = 40
    sets, enc_calls, dec_calls = [], [], []
    for s in range(n_sets):
        rk = synth.tensor_recipe(1, s, "k", D)
        rv = synth.tensor_recipe(1, s, "v", D)
        st = dict(ck=torch.from_numpy(synth.sample_codebook(rk, cfg.c, cfg.b)).cuda(),
                  cv=torch.from_numpy(synth.sample_codebook(rv, cfg.c, cfg.b)).cuda(),
                  xk=synth.sample_activations_torch(rk, T, s, "cuda").view(1, T, D),
                  xv=synth.sample_activations_torch(rv, T, s + 1000, "cuda").view(1, T, D),
                  kcache=cq.alloc_cache(fmt, 1, T), vcache=cq.alloc_cache(fmt, 1, T),
                  q=torch.from_numpy(synth.sample_query(1, s, 1, cfg.n_q_heads, cfg.head_dim)).cuda(),
                  out=torch.empty((1, cfg.n_q_heads, cfg.head_dim), dtype=torch.float16, device="cuda"))
        st["ws"] = torch.empty(max(16, cq.cq_decode_workspace_bytes(fmt, 1, cfg.n_q_heads, T, 0)), dtype=torch.uint8, device="cuda")
        enc_calls.append(cq.prepare_encode_kv(st["xk"], st["xv"], st["ck"], st["cv"], fmt, st["kcache"], st["vcache"], 0, T))
        dec_calls.append(cq.prepare_decode_attention(st["q"], st["kcache"], st["vcache"], st["ck"], st["cv"], scale, fmt, T, T,
                                                     out=st["out"], workspace=st["ws"])[0])
        sets.append(st)
    torch.cuda.synchronize()
    both = []
    for e, d in zip(enc_calls, dec_calls):
        both.append(lambda e=e, d=d: (e(), d()))
    ms_both = time_rotating(torch, both, 5)
    ms_enc = time_rotating(torch, enc_calls, 5)
    ms_dec = time_rotating(torch, dec_calls, 5)
    code_bytes = T * 2 * D * cfg.b // (8 * cfg.c)
    enc_r, enc_pairs = encode_roofline("encode_mfma_kernel<16, 8, 8, 8, true, 1> (K and V in one cq_encode_kv launch)", 2 * T, D, 256, ms_enc, True)
    enc_r.update(achieved=MFMA_SCORE_OPS * enc_pairs / 8 / 1e12, frac=MFMA_SCORE_OPS * enc_pairs / 8 / VALU_PEAK_LANE_OPS)
    out["cfg1_encode_1024_tokens_then_one_decode_step"] = {
        "workload": "CQ-8c8b, batch 1, 32 heads x 128, context 1024: cq_encode_kv of all 1024 tokens (K and V), then "
                    "cq_decode_attention over them; latency of the pair and of each call (launch to launch, rotating sets)",
        "ms_encode_plus_decode": ms_both, "ms_encode_kv": ms_enc, "ms_decode_attention": ms_dec,
        "encode_tokens_per_s_per_tensor": T / (ms_enc * 1e-3) , "decode_kv_tokens_per_s": T / (ms_dec * 1e-3),
        "buffer_sets": n_sets, "cache_resident": False, "bytes_between_reuse": (n_sets - 1) * (code_bytes + 2 * 2 * D * 256 + 2 * 2 * T * D),
        "note": "latency-bound: 1 MiB of codes is 0.13 us of HBM time; the decode launch is one table build and one epilogue",
        "roofline": hbm_roofline(kernel_name(cfg), kernel_name(cfg), code_bytes, ms_dec, 5 * n_sets),
        "roofline_encode": enc_r}
    del sets, enc_calls, dec_calls, both
    torch.cuda.empty_cache()

    # ---- configuration 5: CQ-8c8b, batch 4, context 131072 (the 1-bit-per-channel long-context case)
    cfg, fmt, sets, entry = decode_config_entry(cq, synth, torch, 5, 8, "CQ-8c8b long context")
    out["decode_long_context"] = entry
    B, T, D = cfg.batch, cfg.context, cfg.kv_channels
    code_bytes = B * T * 2 * D * cfg.b // (8 * cfg.c)
    st0 = sets[0]
    # the same call through the entry point that allocates nothing (static scratch for the partials)
    call_s = cq.prepare_decode_attention_static(st0["q"], st0["kcache"], st0["vcache"], st0["ck"], st0["cv"], scale, fmt, T, T, st0["out"])
    calls_s = [cq.prepare_decode_attention_static(s["q"], s["kcache"], s["vcache"], s["ck"], s["cv"], scale, fmt, T, T, s["out"]) for s in sets]
    out["decode_long_context"]["ms_static_scratch_entry_point"] = time_rotating(torch, calls_s, 4)
    del call_s, calls_s
    # its prefill-sized encode: 32768 tokens x 4096 channels, one tensor
    chunk = cfg.encode_tokens
    xk = synth.sample_activations_torch(st0["rk"], chunk, 777, "cuda").view(1, chunk, D)
    scratch_cache = cq.alloc_cache(fmt, 1, chunk)
    enc_ms, _ = time_calls(torch, lambda: cq.cq_encode(xk, st0["ck"], fmt, scratch_cache, 0, chunk), 5, 1)
    enc_r, enc_pairs = encode_roofline("encode_mfma_kernel<16, 8, 8, 4, true, 4>", chunk, D, 256, enc_ms, True)
    enc_r.update(achieved=MFMA_SCORE_OPS * enc_pairs / 8 / 1e12, frac=MFMA_SCORE_OPS * enc_pairs / 8 / VALU_PEAK_LANE_OPS)
    out["encode_prefill"] = {"workload": "CQ-8c8b, 32768 tokens x 4096 channels, one tensor, one cq_encode call",
                             "ms": enc_ms, "tokens_per_s": chunk / (enc_ms * 1e-3), "roofline": enc_r}
    del xk, scratch_cache
    # the same caches read as pre-RoPE keys (query-side rotation; phase K is ALU-bound)
    rope = cq.RopeTable(10000.0, T)
    split_r = cq.cq_decode_rope_default_split(fmt, B, cfg.n_q_heads, T)
    calls_r = []
    for s in sets:
        ws_r = torch.empty(cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, split_r), dtype=torch.uint8, device="cuda")
        calls_r.append(cq.prepare_decode_attention_rope(s["q"], s["kcache"], s["vcache"], s["ck"], s["cv"], scale, fmt, T, T, rope,
                                                        tokens_per_split=split_r, out=s["out"], workspace=ws_r)[0])
    ms_r = time_rotating(torch, calls_r, 3)
    out["decode_long_context_pre_rope_keys"] = {
        "workload": "as decode_long_context, keys cached before RoPE (cq_decode_attention_rope, base 10000)",
        "ms": ms_r, "kv_tokens_per_s": B * T / (ms_r * 1e-3),
        "code_read_GBps": code_bytes / (ms_r * 1e-3) / 1e9, "tokens_per_split": split_r,
        "slowdown_vs_position_independent": ms_r / entry["ms"], "buffer_sets": len(sets), "cache_resident": False,
        "roofline": hbm_roofline("decode_rope_kernel<16, 8, 512, false, 8>", "decode_rope_kernel<16, 8, 512, false, 8>", code_bytes, ms_r,
                                 3 * len(sets),
                                 note="bound by the vector ALU (per-token rotation), not by HBM; the HBM fraction is what the "
                                      "metric asks for"),
        # 6 vector instructions per (token, head, channel pair) is what the rotation and the dot product need
        # (4 mixed-precision multiply-adds with a scalar cosine / sine, 2 plain ones); the peak is one vector
        # instruction per SIMD every 4 cycles
        "roofline_alu": {"bound": "alu", "unit": "T lane-instr/s", "peak": (VALU_PEAK_LANE_OPS / 1e12),
                         "achieved": B * cfg.n_q_heads * T * 64 * 6 / (ms_r * 1e-3) / 1e12,
                         "frac": B * cfg.n_q_heads * T * 64 * 6 / (ms_r * 1e-3) / 1e12 / (VALU_PEAK_LANE_OPS / 1e12),
                         "algorithmic_lane_instructions_per_token_head": 384}}
    del calls_r
    # a prefill chunk over the same caches: the last 512 tokens of each sequence attend causally
    # (cq_chunk_attention on the matrix cores); 4 x 32 x 512 query rows x ~130816 visible tokens each
    m_chunk = 512
    qc = torch.randn((B, m_chunk, cfg.n_q_heads, cfg.head_dim), device="cuda").half()
    call_c, _ = cq.prepare_chunk_attention(qc, st0["kcache"], st0["vcache"], st0["ck"], st0["cv"], scale, fmt, T, T)
    med_c, _ = time_calls(torch, call_c, 4, 1)
    pairs = B * cfg.n_q_heads * sum(T - m_chunk + j + 1 for j in range(m_chunk))
    executed = pairs * 6 * cfg.head_dim / (med_c * 1e-3) / 1e12
    out["chunk_attention_long_context"] = {
        "workload": "CQ-8c8b, batch 4, 32 heads x 128, context 131072: causal attention of the last 512 tokens "
                    "(cq_chunk_attention)",
        "ms": med_c, "query_token_pairs_per_s": pairs / (med_c * 1e-3),
        "useful_TFLOPs": pairs * 4 * cfg.head_dim / (med_c * 1e-3) / 1e12,
        "roofline": {"bound": "mfma", "kernel": "chunk_attention_kernel<16, 8, 8, 8, false>", "achieved": executed, "peak": FP16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": executed / FP16_MFMA_PEAK_TFLOPS, "traffic": None,
                     "note": "executed fp16 MFMA work (probabilities split into two fp16 parts: 6 d flops per pair, 4 d useful)"}}
    # the same chunk over the caches read as pre-RoPE keys: each key tile is rotated once in LDS
    call_cr, _ = cq.prepare_chunk_attention_rope(qc, st0["kcache"], st0["vcache"], st0["ck"], st0["cv"], scale, fmt, T, T, rope)
    med_cr, _ = time_calls(torch, call_cr, 4, 1)
    out["chunk_attention_long_context_pre_rope_keys"] = {
        "workload": "as chunk_attention_long_context, keys cached before RoPE (cq_chunk_attention_rope, base 10000)",
        "ms": med_cr, "query_token_pairs_per_s": pairs / (med_cr * 1e-3), "slowdown_vs_position_independent": med_cr / med_c,
        "roofline": {"bound": "mfma", "kernel": "chunk_attention_kernel<16, 8, 8, 8, true>",
                     "achieved": pairs * 6 * cfg.head_dim / (med_cr * 1e-3) / 1e12, "peak": FP16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": pairs * 6 * cfg.head_dim / (med_cr * 1e-3) / 1e12 / FP16_MFMA_PEAK_TFLOPS, "traffic": None}}
    del qc, call_c, call_cr, sets, st0
    torch.cuda.empty_cache()

    # ---- configurations 3 and 4
    for cfg_id, key, label in ((3, "decode_cq2c8b_batch64_ctx8192", "CQ-2c8b"),
                               (4, "decode_cq8c10b_gqa_batch32_ctx16384", "CQ-8c10b, grouped queries")):
        cfg, fmt, sets, entry = decode_config_entry(cq, synth, torch, cfg_id, 6, label)
        if cfg_id == 4:
            entry["binding_ceiling"] = ("not HBM: per workgroup the score table and the epilogue each walk a 256 KB codebook "
                                        "(L2) against 640 KB of codes, and the four query heads of a KV head repeat both")
        out[key] = entry
        if cfg.encode_tokens > 1:           # the configuration's prefill chunk: B x encode_tokens tokens, one tensor
            B, T, D, te = cfg.batch, cfg.context, cfg.kv_channels, cfg.encode_tokens
            x = synth.sample_activations_torch(sets[0]["rk"], B * te, 4242, "cuda").view(B, te, D)
            enc_ms, _ = time_calls(torch, lambda: cq.cq_encode(x, sets[0]["ck"], fmt, sets[0]["kcache"], 0, T), 5, 1)
            gh = cfg.head_dim // cfg.c
            enc_r, enc_pairs = encode_roofline((f"encode_mfma_kernel<{gh}, {cfg.c}, {cfg.b}, 4, true, 4>" if cfg.b == 8 else f"encode_mfma_kernel<{gh}, {cfg.c}, {cfg.b}, 4, false, 1>"), B * te, D, 1 << cfg.b, enc_ms, True)
            enc_r.update(achieved=MFMA_SCORE_OPS * enc_pairs / cfg.c / 1e12, frac=MFMA_SCORE_OPS * enc_pairs / cfg.c / VALU_PEAK_LANE_OPS)
            out[f"encode_cq{cfg.c}c{cfg.b}b_{B}x{te}"] = {
                "workload": f"CQ-{cfg.c}c{cfg.b}b, {B} sequences x {te} tokens x {D} channels, one tensor, one cq_encode call",
                "ms": enc_ms, "tokens_per_s": B * te / (enc_ms * 1e-3), "roofline": enc_r}
            del x
        del sets
        torch.cuda.empty_cache()

    # ---- grouped queries over keys cached before RoPE: four query heads of a KV head share every key rotation
    # (Mistral-like 32 / 8 heads, CQ-8c8b, batch 32, context 16384; uniform random codes; three cache sets)
    fmt_g = cq.CQFormat(8, 8, 128, 8)
    Bg, Tg, Hq_g = 32, 16384, 32
    code_bytes_g = Bg * Tg * 2 * fmt_g.channels * 8 // 64
    rope_g = cq.RopeTable(10000.0, Tg)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    qg = torch.randn((Bg, Hq_g, 128), device="cuda", generator=gen).half()
    shared_calls, per_head_calls = [], []
    split_g = cq.cq_decode_rope_default_split(fmt_g, Bg, Hq_g, Tg)
    keep = []
    for _ in range(3):
        nb = cq.cq_cache_bytes(fmt_g, Bg, Tg)
        kc_ = torch.randint(0, 256, (nb,), dtype=torch.uint8, device="cuda", generator=gen)
        vc_ = torch.randint(0, 256, (nb,), dtype=torch.uint8, device="cuda", generator=gen)
        ck_ = torch.randn((fmt_g.groups, 256, 8), device="cuda", generator=gen).half()
        cv_ = torch.randn((fmt_g.groups, 256, 8), device="cuda", generator=gen).half()
        keep.append((kc_, vc_, ck_, cv_))
        shared_calls.append(cq.prepare_decode_attention_rope(qg, kc_, vc_, ck_, cv_, 0.088, fmt_g, Tg, Tg, rope_g, tokens_per_split=split_g)[0])
        per_head_calls.append(cq.prepare_decode_attention_rope(qg, kc_, vc_, ck_, cv_, 0.088, fmt_g, Tg, Tg, rope_g, tokens_per_split=Tg)[0])
    ms_sh, ms_ph = (time_rotating(torch, c, 3) for c in (shared_calls, per_head_calls))
    out["decode_gqa_pre_rope_keys_cq8c8b_batch32_ctx16384"] = {
        "workload": "CQ-8c8b, 32 query / 8 KV heads, batch 32, context 16384, keys cached before RoPE (cq_decode_attention_rope): "
                    "one workgroup rotates every key once for the four query heads of its KV head",
        "ms": ms_sh, "tokens_per_split": split_g, "kv_tokens_per_s": Bg * Tg / (ms_sh * 1e-3),
        "ms_one_query_head_per_workgroup": ms_ph, "speedup_from_sharing": ms_ph / ms_sh,
        "buffer_sets": 3, "cache_resident": False,
        "roofline": hbm_roofline("decode_rope_gqa_kernel<16, 8, 512, false>", "decode_rope_gqa_kernel<16, 8, 512, false>", code_bytes_g, ms_sh, 9,
                                 note="bound by vector and matrix instruction issue (per channel pair 4 vector + 2 matrix "
                                      "instructions for four heads), not by HBM")}
    del keep, shared_calls, per_head_calls, qg
    torch.cuda.empty_cache()

    # ---- centroid learning on a calibration tensor of the paper's size (16 sequences x 2048 tokens):
    # k-means++ and 100 Lloyd iterations for each of the 512 groups of one CQ-8c8b tensor
    cfg = synth.CONFIGS[5]
    fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
    D = cfg.kv_channels
    rk = synth.tensor_recipe(5, 0, "k", D)
    n_cal, iters = 16 * 2048, 100
    xcal = synth.sample_activations_torch(rk, n_cal, 977, "cuda").view(n_cal, D)
    g = torch.Generator(device="cuda")
    g.manual_seed(240503917)
    rnd = torch.randint(-2 ** 63, 2 ** 63 - 1, (fmt.groups, 1 << cfg.b), dtype=torch.int64, device="cuda", generator=g)
    wsk = torch.empty(cq.cq_kmeans_workspace_bytes(fmt, n_cal), dtype=torch.uint8, device="cuda")
    init_ms, _ = time_calls(torch, lambda: cq.cq_kmeans_fit(xcal, fmt, 0, rnd=rnd, workspace=wsk), 3, 1)
    fit_ms, _ = time_calls(torch, lambda: cq.cq_kmeans_fit(xcal, fmt, iters, rnd=rnd, workspace=wsk), 3, 1)
    per_iter = (fit_ms - init_ms) / iters
    pairs_iter = n_cal * fmt.groups * 256
    out["centroid_learning"] = {
        "workload": "CQ-8c8b, 32768 calibration tokens x 4096 channels, one tensor: k-means++ then 100 Lloyd "
                    "iterations in each of 512 groups (cq_kmeans_fit)",
        "ms": fit_ms, "kmeanspp_ms": init_ms, "ms_per_iteration": per_iter,
        "seconds_for_64_tensors": fit_ms * 64 / 1e3,
        "roofline": {"bound": "alu", "kernel": "kmeans_assign_kernel + kmeans_update_kernel, per iteration (fp32 subtract, multiply, "
                                               "add per (token channel, centroid) pair: 3 flops)",
                     "achieved": 3 * 8 * pairs_iter / (per_iter * 1e-3) / 1e12, "peak": FP32_VECTOR_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": 3 * 8 * pairs_iter / (per_iter * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, "traffic": None}}
    return out


def cpu_baseline(synth, cfg, budget_s=12.0):
    """The fp64 oracle, as it stands, on this host's cores: one layer-step (encode the new rows,
    attend over the context) for a sub-batch sized to the time budget."""
    import numpy as np
    from oracle import cq_oracle as O
    cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1000000")))
    O.set_threads(cores)
    D, T = cfg.kv_channels, cfg.context
    rk = synth.tensor_recipe(cfg.cfg_id, 0, "k", D)
    rv = synth.tensor_recipe(cfg.cfg_id, 0, "v", D)
    ck, cv = synth.sample_codebook(rk, cfg.c, cfg.b), synth.sample_codebook(rv, cfg.c, cfg.b)
    rng = np.random.default_rng(0)
    # probe with one sequence, then scale the sub-batch
    def one(bs):
        kc = rng.integers(0, 1 << cfg.b, size=(bs, T, cfg.n_groups)).astype(np.uint16)
        vc = rng.integers(0, 1 << cfg.b, size=(bs, T, cfg.n_groups)).astype(np.uint16)
        xk = np.stack([synth.sample_activations(rk, 1, chunk=1000 + n) for n in range(bs)])
        xv = np.stack([synth.sample_activations(rv, 1, chunk=1000 + n) for n in range(bs)])
        q = synth.sample_query(cfg.cfg_id, 0, bs, cfg.n_q_heads, cfg.head_dim)
        t0 = time.perf_counter()
        kc[:, T - 1] = O.encode(xk[:, 0], ck)
        vc[:, T - 1] = O.encode(xv[:, 0], cv)
        O.attention(q, kc, vc, ck, cv, 1.0 / math.sqrt(cfg.head_dim), cfg.n_kv_heads)
        return time.perf_counter() - t0
    t1 = one(1)
    bs = int(max(1, min(cfg.batch, budget_s / max(t1, 1e-3))))
    # one pass of the sub-batch measures its real cost (sequences run in parallel); repeat it up to
    # the budget
    t_first = one(bs)
    reps = 1 + int(max(0, min(63, (budget_s - t_first) / max(t_first, 1e-3))))
    t = t_first + sum(one(bs) for _ in range(reps - 1))
    return {"value": reps * bs * T / t, "unit": "KV tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} layer-step(s) (2 x encode of {bs} new rows + attention over {T} cached tokens) "
                      f"for {bs} of {cfg.batch} sequences, {t:.1f} s in total; random codes in the cache",
            "threads_env": os.environ.get("OMP_NUM_THREADS")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debug only)")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations and entry points")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only-extra", action="store_true", help="(profiling aid) run only the `extra` measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    import paper_2405_03917_amd as cq
    import synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    cq.load()
    torch.cuda.set_device(0)
    if args.only_extra:
        print(json.dumps({"extra": extra_measurements(cq, synth, torch)}), flush=True)
        return
    cfg = synth.CONFIGS[2]
    n_layers = args.layers or cfg.layers
    scale = 1.0 / math.sqrt(cfg.head_dim)

    t_setup = time.perf_counter()
    fmt, t_cap, layers = build_workload(cq, synth, torch, cfg, n_layers)
    torch.cuda.synchronize()
    log(f"[bench] setup {time.perf_counter() - t_setup:.1f} s")

    prepare_calls(cq, fmt, cfg, t_cap, layers, scale)
    for _ in range(max(1, args.warmup)):
        run_step(layers)
    torch.cuda.synchronize()

    # capture the step (one launch per layer) in a HIP graph on a side stream
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_step(layers)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_step(layers)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps between a HIP event pair on the launching stream and a
    # host clock read on both sides of a synchronize.  Headline: 32 prepared calls per step in
    # stream order.  The same steps as replays of the captured graph are reported beside it.
    def timed(step_fn):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(args.steps):
            step_fn()
        ev1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1)
    dt, ev_ms = timed(lambda: run_step(layers))
    dt_graph, _ = timed(graph.replay)
    # the same step as ONE launch over all layers (possible because the workload's layers are
    # independent; reported beside the headline, which stays with one launch per layer)
    table = cq.LayerTable([dict(q=st.q, x_k_new=st.xk_new[:, 0, :], x_v_new=st.xv_new[:, 0, :], k_codes=st.kcache,
                                v_codes=st.vcache, k_centroids=st.ck, v_centroids=st.cv, out=st.out) for st in layers],
                          fmt, t_cap)
    step_all = cq.prepare_decode_step_layers(table, scale, cfg.context)
    for _ in range(max(1, args.warmup)):
        step_all()
    dt_layers, _ = timed(step_all)
    ms_per_step = dt / args.steps * 1e3
    kv_tokens = cfg.batch * cfg.context * n_layers
    value = kv_tokens / (dt / args.steps)
    log(f"[bench] stream-order launches {ms_per_step:.3f} ms/step, graph replay {dt_graph / args.steps * 1e3:.3f} ms/step "
        f"-> {value:.3e} KV tokens/s")

    # mean duration of one launch over the timed region (one launch per layer; the gap between
    # consecutive launches is included)
    dec_ms = ev_ms / (args.steps * n_layers)
    code_bytes = cfg.batch * cfg.context * 2 * cfg.kv_channels * cfg.b // (8 * cfg.c)   # per launch
    kname = kernel_name(cfg, step=True)
    roofline = hbm_roofline(kname + " (cq_decode_step; one launch = one layer)", kname, code_bytes, dec_ms, args.steps * n_layers)
    log(f"[bench] step kernel avg {dec_ms * 1e3:.1f} us launch to launch -> {roofline['achieved']:.0f} GB/s of code reads "
        f"({100 * roofline['frac']:.1f}% of 8 TB/s)")

    # the two-launch form of the step, and plain decode attention alone, for comparison
    unf_med, _ = time_calls(torch, lambda: run_step_unfused(layers), 5, 1)
    def dec_all():
        for st in layers:
            st.dec()
    dec_only_ms, _ = time_calls(torch, dec_all, 5, 1)
    dec_only_ms /= len(layers)

    # yardsticks: a read-only streaming kernel (one launch over 2 GiB) and a plain copy kernel of
    # known size (256 MiB; its HBM counters calibrate the decode kernel's)
    sink = torch.zeros(8192, dtype=torch.uint8, device="cuda")
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    big.zero_()
    probe_med, _ = time_calls(torch, lambda: cq.cq_probe_stream_read(big, sink), 10, 2)
    stream_gbps = big.numel() / (probe_med * 1e-3) / 1e9
    half = 256 << 20
    copy_med, _ = time_calls(torch, lambda: cq.cq_probe_copy(big[:half], big[half:2 * half]), 5, 1)
    del big
    roofline["stream_read_GBps"] = stream_gbps
    roofline["frac_of_stream_read"] = roofline["achieved"] / stream_gbps
    roofline["copy_256MiB_GBps_read_plus_write"] = 2 * half / (copy_med * 1e-3) / 1e9
    log(f"[bench] streaming-read yardstick: {stream_gbps:.0f} GB/s; decode kernel at {100 * roofline['achieved'] / stream_gbps:.1f}% of it; "
        f"copy {roofline['copy_256MiB_GBps_read_plus_write']:.0f} GB/s (read+write)")

    # encode share of the step (same launches, events around the two encodes of each layer)
    def enc_all():
        for st in layers:
            st.enc_kv()
    enc_med, _ = time_calls(torch, enc_all, 10, 2)
    enc_med /= len(layers)
    enc_r, enc_pairs = encode_roofline("encode_centroids_kernel<32, 4, 8> (K and V rows in one launch)", 2 * cfg.batch,
                                       cfg.kv_channels, 256, enc_med, False)
    enc_r.update(achieved=(2 * cfg.c + 3) * enc_pairs / cfg.c / 1e12, frac=(2 * cfg.c + 3) * enc_pairs / cfg.c / VALU_PEAK_LANE_OPS,
                 note="launch- and latency-bound: 32 rows against a 2 x 2 MiB codebook; the fused step hides it")
    result = {
        "metric": METRIC, "value": value, "unit": "KV tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "dtype_note": "fp16 inputs (activations, queries, centroids) and fp16 output; lookup tables, scores, softmax and "
                      "accumulation in fp32; probability bins in 32-bit fixed point",
        "config": {"workload": "CQ-4c8b decode step, 32 layers, batch 16, 32 heads x 128, context 4096, MHA; "
                               "per layer: one cq_decode_step launch = encode 16 new K rows + 16 new V rows, then decode attention",
                   "format": "CQ-4c8b", "batch": cfg.batch, "context": cfg.context, "layers": n_layers,
                   "launch": "32 prepared calls in stream order", "tokens_per_split":
                       cq.cq_decode_default_split(fmt, cfg.batch, cfg.n_q_heads, cfg.context)},
        "roofline": roofline,
        "hbm_code_read_GBps_whole_step": kv_tokens * 2 * cfg.kv_channels * cfg.b // (8 * cfg.c) / (dt / args.steps) / 1e9,
        "stream_order_ms_per_step": ms_per_step, "graph_replay_ms_per_step": dt_graph / args.steps * 1e3,
        "unfused_eager_ms_per_step": unf_med,
        "layer_batched_launch_ms_per_step": dt_layers / args.steps * 1e3,
        "decode_attention_only": {"workload": "cq_decode_attention of one layer (no fused encode), eager back-to-back "
                                              "launches over the 32 layers' caches, HIP events", "ms": dec_only_ms,
                                  "code_read_GBps": code_bytes / (dec_only_ms * 1e-3) / 1e9, "buffer_sets": n_layers,
                                  "cache_resident": False,
                                  "roofline": hbm_roofline(kernel_name(cfg), kernel_name(cfg), code_bytes, dec_only_ms, 5 * n_layers)},
        "encode_decode_step": {"workload": "16 new K rows + 16 new V rows x 4096 channels, one cq_encode_kv launch "
                                           "(mean over 32 back-to-back launches)", "ms": enc_med,
                               "tokens_per_s_per_tensor": cfg.batch / (enc_med * 1e-3), "roofline": enc_r},
    }
    del graph, table, step_all
    if not args.no_extra:
        del layers
        torch.cuda.empty_cache()
        try:
            result["extra"] = extra_measurements(cq, synth, torch)
            log(f"[bench] extra: {json.dumps(result['extra'])}")
        except Exception as e:      # side measurements must not lose the main line
            result["extra"] = {"error": repr(e)}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(synth, cfg)
        log(f"[bench] cpu oracle: {result['cpu_baseline']}")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
