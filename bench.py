#!/usr/bin/env python3
"""Throughput of the CQ hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

Workload (the second named configuration): CQ-4c8b (2 bits per channel) on a Llama-2-7B-shaped
KV cache -- 32 layers, batch 16, 32 heads x 128, context 4096, MHA.  One STEP is one decode step
of the whole hot path over all 32 layers: per layer, encode the 16 new key rows and the 16 new
value rows into cache position 4095 and attend over all 4096 cached tokens -- one fused
cq_decode_step launch, bit-identical to cq_encode_kv followed by cq_decode_attention.  Every layer has its own codebooks, caches, queries and new rows (4 GiB of
codes in total, far more than the 256 MB Infinity Cache, so code reads are real HBM reads).

Inputs are synthetic and resident in HBM before the timed region: correlated-Gaussian K/V rows
(synth/generator.py) drawn on the device and REALLY encoded with cq_encode to fill the caches.

The timed region replays a HIP graph of the step (32 kernel launches) K times between two
synchronisations.  After it, the same launches are run eagerly with a HIP event pair around
every cq_decode_step call to obtain the kernel's own average duration (with a single context
split, as here, that call is exactly one kernel).

One JSON line is printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published peak, GB/s
# HBM bytes per launch of the fused decode-step kernel from rocprofv3 counters (FETCH_SIZE x 1.9998
# + WRITE_SIZE, KiB per dispatch), see profiles/decode_step_kernel_cq4c8b_batch16_ctx4096.md
TRAFFIC_BYTES_PER_LAUNCH = (67945.9 * 1.9998 + 192.0) * 1024
METRIC = "decode-attn KV tokens/s & achieved HBM GB/s (% peak); cq_encode tokens/s"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class LayerState:
    """Device buffers of one layer."""
    __slots__ = ("ck", "cv", "kcache", "vcache", "q", "xk_new", "xv_new", "out", "ws", "enc_kv", "dec", "step")


def build_workload(cq, synth, torch, cfg, n_layers, fill_chunk_tokens=16384):
    """Allocate and fill every layer's buffers.  Cache positions 0 .. T-2 come from encoding
    device-generated activations; the last position is written by the timed step itself."""
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
        import numpy as np
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


def run_step(layers, events=None):
    """One decode step: per layer ONE cq_decode_step launch (encode the new K/V rows of the 16
    sequences into position T-1, then attend over all T positions)."""
    for i, st in enumerate(layers):
        if events is not None:
            events[i][0].record()
        st.step()
        if events is not None:
            events[i][1].record()


def run_step_unfused(layers):
    """The same step as two launches per layer (cq_encode_kv, cq_decode_attention)."""
    for st in layers:
        st.enc_kv()
        st.dec()


def time_calls(torch, fn, iters, warmup=2):
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


def extra_measurements(cq, synth, torch):
    """Decode attention at 1 bit per channel on a long context (CQ-8c8b, batch 4, 131072 tokens)
    and prefill-sized cq_encode (32768 tokens): the cases the headline targets are quoted on."""
    import numpy as np
    out = {}
    cfg = synth.CONFIGS[5]
    fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
    B, T, D = cfg.batch, cfg.context, cfg.kv_channels
    rk = synth.tensor_recipe(5, 0, "k", D)
    rv = synth.tensor_recipe(5, 0, "v", D)
    ck = torch.from_numpy(synth.sample_codebook(rk, cfg.c, cfg.b)).cuda()
    cv = torch.from_numpy(synth.sample_codebook(rv, cfg.c, cfg.b)).cuda()
    kcache, vcache = cq.alloc_cache(fmt, B, T), cq.alloc_cache(fmt, B, T)
    per_seq = kcache.numel() // B
    chunk = cfg.encode_tokens
    enc_ms = None
    for n in range(B):
        for t0 in range(0, T, chunk):
            xk = synth.sample_activations_torch(rk, chunk, 31 * n + t0, "cuda").view(1, chunk, D)
            xv = synth.sample_activations_torch(rv, chunk, 31 * n + t0 + 1, "cuda").view(1, chunk, D)
            if enc_ms is None:      # time the 32768-token prefill encode once (per tensor)
                enc_ms, _ = time_calls(torch, lambda: cq.cq_encode(xk, ck, fmt, kcache[:per_seq], 0, T), 5, 1)
            cq.cq_encode(xk, ck, fmt, kcache[n * per_seq:(n + 1) * per_seq], t0, T)
            cq.cq_encode(xv, cv, fmt, vcache[n * per_seq:(n + 1) * per_seq], t0, T)
            del xk, xv
    torch.cuda.synchronize()
    out["encode_prefill"] = {"workload": "CQ-8c8b, 32768 tokens x 4096 channels, one tensor",
                             "ms": enc_ms, "tokens_per_s": chunk / (enc_ms * 1e-3)}
    q = torch.from_numpy(synth.sample_query(5, 0, B, cfg.n_q_heads, cfg.head_dim)).cuda()
    o = torch.empty((B, cfg.n_q_heads, cfg.head_dim), dtype=torch.float16, device="cuda")
    ws = torch.empty(cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, 0), dtype=torch.uint8, device="cuda")
    scale = 1.0 / math.sqrt(cfg.head_dim)
    med, mean = time_calls(torch, lambda: cq.cq_decode_attention(q, kcache, vcache, ck, cv, scale, fmt, T, T,
                                                                 out=o, workspace=ws), 20, 3)
    code_bytes = B * T * 2 * D * cfg.b // (8 * cfg.c)
    out["decode_long_context"] = {
        "workload": "CQ-8c8b, batch 4, 32 heads x 128, context 131072, one layer (split kernel + merge)",
        "ms": med, "kv_tokens_per_s": B * T / (med * 1e-3),
        "code_read_GBps": code_bytes / (med * 1e-3) / 1e9,
        "frac_of_hbm_peak": code_bytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "tokens_per_split": cq.cq_decode_default_split(fmt, B, cfg.n_q_heads, T)}
    # the same caches read as pre-RoPE keys (query-side rotation; phase K is ALU-bound)
    rope = cq.RopeTable(10000.0, T)
    split_r = cq.cq_decode_rope_default_split(fmt, B, cfg.n_q_heads, T)
    ws_r = torch.empty(cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, split_r), dtype=torch.uint8, device="cuda")
    call_r, _ = cq.prepare_decode_attention_rope(q, kcache, vcache, ck, cv, scale, fmt, T, T, rope,
                                                 tokens_per_split=split_r, out=o, workspace=ws_r)
    med_r, _ = time_calls(torch, call_r, 10, 2)
    out["decode_long_context_pre_rope_keys"] = {
        "workload": "as decode_long_context, keys cached before RoPE (cq_decode_attention_rope, base 10000)",
        "ms": med_r, "kv_tokens_per_s": B * T / (med_r * 1e-3),
        "code_read_GBps": code_bytes / (med_r * 1e-3) / 1e9, "tokens_per_split": split_r,
        "slowdown_vs_position_independent": med_r / med}
    # a prefill chunk over the same caches: the last 512 tokens of each sequence attend causally
    # (cq_chunk_attention on the matrix cores); 4 x 32 x 512 query rows x ~130816 visible tokens each
    m_chunk = 512
    qc = torch.randn((B, m_chunk, cfg.n_q_heads, cfg.head_dim), device="cuda").half()
    call_c, _ = cq.prepare_chunk_attention(qc, kcache, vcache, ck, cv, scale, fmt, T, T)
    med_c, _ = time_calls(torch, call_c, 5, 1)
    pairs = B * cfg.n_q_heads * sum(T - m_chunk + j + 1 for j in range(m_chunk))
    out["chunk_attention_long_context"] = {
        "workload": "CQ-8c8b, batch 4, 32 heads x 128, context 131072: causal attention of the last 512 tokens "
                    "(cq_chunk_attention)",
        "ms": med_c, "query_token_pairs_per_s": pairs / (med_c * 1e-3),
        "useful_TFLOPs": pairs * 4 * cfg.head_dim / (med_c * 1e-3) / 1e12,
        "mfma_TFLOPs_executed": pairs * 6 * cfg.head_dim / (med_c * 1e-3) / 1e12,
        "frac_of_fp16_mfma_peak_executed": pairs * 6 * cfg.head_dim / (med_c * 1e-3) / 1e12 / 2500.0}
    del kcache, vcache, qc
    # centroid learning on a calibration tensor of the paper's size (16 sequences x 2048 tokens):
    # k-means++ and 100 Lloyd iterations for each of the 512 groups of one CQ-8c8b tensor
    n_cal, iters = 16 * 2048, 100
    xcal = synth.sample_activations_torch(rk, n_cal, 977, "cuda").view(n_cal, D)
    g = torch.Generator(device="cuda")
    g.manual_seed(240503917)
    rnd = torch.randint(-2 ** 63, 2 ** 63 - 1, (fmt.groups, 1 << cfg.b), dtype=torch.int64, device="cuda", generator=g)
    wsk = torch.empty(cq.cq_kmeans_workspace_bytes(fmt, n_cal), dtype=torch.uint8, device="cuda")
    init_ms, _ = time_calls(torch, lambda: cq.cq_kmeans_fit(xcal, fmt, 0, rnd=rnd, workspace=wsk), 3, 1)
    fit_ms, _ = time_calls(torch, lambda: cq.cq_kmeans_fit(xcal, fmt, iters, rnd=rnd, workspace=wsk), 3, 1)
    out["centroid_learning"] = {
        "workload": "CQ-8c8b, 32768 calibration tokens x 4096 channels, one tensor: k-means++ then 100 Lloyd "
                    "iterations in each of 512 groups (cq_kmeans_fit)",
        "ms": fit_ms, "kmeanspp_ms": init_ms, "ms_per_iteration": (fit_ms - init_ms) / iters,
        "seconds_for_64_tensors": fit_ms * 64 / 1e3}
    return out


def config_measurements(cq, synth, torch):
    """The other two decode workloads of the named configurations, on caches filled by really
    encoding generated activations: CQ-2c8b (batch 64, context 8192; also its 64 x 512-token
    prefill encode) and CQ-8c10b with grouped queries (32 query / 8 KV heads, batch 32, context
    16384)."""
    out = {}
    for cfg_id, key in ((3, "decode_cq2c8b_batch64_ctx8192"), (4, "decode_cq8c10b_gqa_batch32_ctx16384")):
        cfg = synth.CONFIGS[cfg_id]
        fmt = cq.CQFormat(cfg.c, cfg.b, cfg.head_dim, cfg.n_kv_heads)
        B, T, D = cfg.batch, cfg.context, cfg.kv_channels
        rk = synth.tensor_recipe(cfg_id, 0, "k", D)
        rv = synth.tensor_recipe(cfg_id, 0, "v", D)
        ck = torch.from_numpy(synth.sample_codebook(rk, cfg.c, cfg.b)).cuda()
        cv = torch.from_numpy(synth.sample_codebook(rv, cfg.c, cfg.b)).cuda()
        kcache, vcache = cq.alloc_cache(fmt, B, T), cq.alloc_cache(fmt, B, T)
        per_seq = kcache.numel() // B
        for n in range(B):                  # one sequence per call: T tokens x D channels
            xk = synth.sample_activations_torch(rk, T, 17 * n, "cuda").view(1, T, D)
            xv = synth.sample_activations_torch(rv, T, 17 * n + 1, "cuda").view(1, T, D)
            cq.cq_encode_kv(xk, xv, ck, cv, fmt, kcache[n * per_seq:(n + 1) * per_seq],
                            vcache[n * per_seq:(n + 1) * per_seq], 0, T)
            del xk, xv
        torch.cuda.synchronize()
        q = torch.from_numpy(synth.sample_query(cfg_id, 0, B, cfg.n_q_heads, cfg.head_dim)).cuda()
        o = torch.empty((B, cfg.n_q_heads, cfg.head_dim), dtype=torch.float16, device="cuda")
        ws = torch.empty(max(16, cq.cq_decode_workspace_bytes(fmt, B, cfg.n_q_heads, T, 0)), dtype=torch.uint8, device="cuda")
        scale = 1.0 / math.sqrt(cfg.head_dim)
        call, _ = cq.prepare_decode_attention(q, kcache, vcache, ck, cv, scale, fmt, T, T, out=o, workspace=ws)
        med, _ = time_calls(torch, call, 30, 10)
        code_bytes = B * T * 2 * D * cfg.b // (8 * cfg.c)
        out[key] = {"workload": f"{cfg.name}: cq_decode_attention of one layer, {cfg.n_q_heads} query / {cfg.n_kv_heads} KV heads "
                                "(the codes are larger than the 256 MB last-level cache only for CQ-2c8b)",
                    "ms": med, "kv_tokens_per_s": B * T / (med * 1e-3),
                    "code_read_GBps": code_bytes / (med * 1e-3) / 1e9,
                    "frac_of_hbm_peak": code_bytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                    "tokens_per_split": cq.cq_decode_default_split(fmt, B, cfg.n_q_heads, T)}
        if cfg.encode_tokens > 1:           # the configuration's prefill chunk: B x encode_tokens tokens, one tensor
            te = cfg.encode_tokens
            x = synth.sample_activations_torch(rk, B * te, 4242, "cuda").view(B, te, D)
            enc_ms, _ = time_calls(torch, lambda: cq.cq_encode(x, ck, fmt, kcache, 0, T), 5, 1)
            out[f"encode_cq{cfg.c}c{cfg.b}b_{B}x{te}"] = {
                "workload": f"CQ-{cfg.c}c{cfg.b}b, {B} sequences x {te} tokens x {D} channels, one tensor, one cq_encode call",
                "ms": enc_ms, "tokens_per_s": B * te / (enc_ms * 1e-3)}
            del x
        del kcache, vcache
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debug only)")
    ap.add_argument("--no-extra", action="store_true", help="skip the long-context / prefill side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
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

    # capture the step (3 * layers launches) in a HIP graph on a side stream
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
    # host clock read on both sides of a synchronize.  The step is timed twice, launched as a
    # replay of the captured graph and as 32 prepared calls in stream order; the faster way of
    # launching the same kernels is the reported one (both are printed).
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
    dt_graph, ev_graph = timed(graph.replay)
    dt_eager, ev_eager = timed(lambda: run_step(layers))
    # the same step as ONE launch over all layers (possible because the workload's layers are
    # independent; reported beside the headline, which stays with one launch per layer)
    table = cq.LayerTable([dict(q=st.q, x_k_new=st.xk_new[:, 0, :], x_v_new=st.xv_new[:, 0, :], k_codes=st.kcache,
                                v_codes=st.vcache, k_centroids=st.ck, v_centroids=st.cv, out=st.out) for st in layers],
                          fmt, t_cap)
    step_all = cq.prepare_decode_step_layers(table, scale, cfg.context)
    step_all()
    dt_layers, _ = timed(step_all)
    launch_mode = "HIP graph of 1 launch per layer" if dt_graph <= dt_eager else "32 prepared calls in stream order"
    dt, ev_ms = (dt_graph, ev_graph) if dt_graph <= dt_eager else (dt_eager, ev_eager)
    ms_per_step = dt / args.steps * 1e3
    kv_tokens = cfg.batch * cfg.context * n_layers
    value = kv_tokens / (dt / args.steps)
    log(f"[bench] graph replay {dt_graph / args.steps * 1e3:.3f} ms/step, stream-order launches "
        f"{dt_eager / args.steps * 1e3:.3f} ms/step -> {value:.3e} KV tokens/s ({launch_mode})")

    # mean duration of one launch over the timed region (one launch per layer; the few hundred
    # nanoseconds of dispatch between back-to-back graph nodes are included)
    dec_ms = ev_ms / (args.steps * n_layers)
    code_bytes = cfg.batch * cfg.context * 2 * cfg.kv_channels * cfg.b // (8 * cfg.c)   # per launch
    achieved = code_bytes / (dec_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_split_kernel<32,4,8,512,true,false,false> (cq_decode_step; one launch = one layer)",
                "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                "traffic": TRAFFIC_BYTES_PER_LAUNCH if n_layers == cfg.layers else None,
                "algorithmic_bytes_per_launch": code_bytes, "avg_launch_ms": dec_ms,
                "launches_timed": args.steps * n_layers}
    log(f"[bench] step kernel avg {dec_ms * 1e3:.1f} us -> {achieved:.0f} GB/s of code reads "
        f"({100 * achieved / HBM_PEAK_GBPS:.1f}% of 8 TB/s)")

    # eager launches of the same step, and of its two-launch form, for comparison
    unf_med, _ = time_calls(torch, lambda: run_step_unfused(layers), 5, 1)
    # plain decode attention alone (no fused encode), back to back over the 32 layers
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
    roofline["frac_of_stream_read"] = achieved / stream_gbps
    roofline["copy_256MiB_GBps_read_plus_write"] = 2 * half / (copy_med * 1e-3) / 1e9
    log(f"[bench] streaming-read yardstick: {stream_gbps:.0f} GB/s; decode kernel at {100 * achieved / stream_gbps:.1f}% of it; "
        f"copy {roofline['copy_256MiB_GBps_read_plus_write']:.0f} GB/s (read+write)")

    # encode share of the step (same launches, events around the two encodes of each layer)
    def enc_all():
        for st in layers:
            st.enc_kv()
    enc_med, _ = time_calls(torch, enc_all, 10, 2)
    enc_med /= len(layers)
    result = {
        "metric": METRIC, "value": value, "unit": "KV tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "CQ-4c8b decode step, 32 layers, batch 16, 32 heads x 128, context 4096, MHA; "
                               "per layer: one cq_decode_step launch = encode 16 new K rows + 16 new V rows, then decode attention",
                   "format": "CQ-4c8b", "batch": cfg.batch, "context": cfg.context, "layers": n_layers,
                   "launch": launch_mode, "tokens_per_split":
                       cq.cq_decode_default_split(fmt, cfg.batch, cfg.n_q_heads, cfg.context)},
        "roofline": roofline,
        "hbm_code_read_GBps_whole_step": kv_tokens * 2 * cfg.kv_channels * cfg.b // (8 * cfg.c) / (dt / args.steps) / 1e9,
        "graph_replay_ms_per_step": dt_graph / args.steps * 1e3,
        "stream_order_ms_per_step": dt_eager / args.steps * 1e3, "unfused_eager_ms_per_step": unf_med,
        "layer_batched_launch_ms_per_step": dt_layers / args.steps * 1e3,
        "decode_attention_only": {"workload": "cq_decode_attention of one layer (no fused encode), eager back-to-back "
                                              "launches, HIP events", "ms": dec_only_ms,
                                  "code_read_GBps": code_bytes / (dec_only_ms * 1e-3) / 1e9},
        "encode_decode_step": {"workload": "16 new K rows + 16 new V rows x 4096 channels, one cq_encode_kv launch "
                                           "(mean over 32 back-to-back launches)", "ms": enc_med,
                               "tokens_per_s_per_tensor": cfg.batch / (enc_med * 1e-3)},
    }
    del graph
    if not args.no_extra:
        del layers
        torch.cuda.empty_cache()
        try:
            result["extra"] = extra_measurements(cq, synth, torch)
            torch.cuda.empty_cache()
            result["extra"].update(config_measurements(cq, synth, torch))
            log(f"[bench] extra: {json.dumps(result['extra'])}")
        except Exception as e:      # side measurements must not lose the main line
            result["extra"] = {"error": repr(e)}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(synth, cfg)
        log(f"[bench] cpu oracle: {result['cpu_baseline']}")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
