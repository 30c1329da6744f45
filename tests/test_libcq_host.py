"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
public header declares, its sizing helpers agree with the paper's densities and with the numpy
restatement of the layout, and every argument-validation path returns before any launch."""
import ctypes
import os
import re

import pytest

import paper_2405_03917_amd as cq
from oracle import code_layout as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "libcq.h")

FORMATS = [(8, 8), (4, 8), (2, 8), (8, 10)]


def _declared():
    text = open(HEADER).read()
    return re.findall(r"CQ_API\s+[\w\s\*]+?\b(cq_\w+)\s*\(", text)


def test_library_loads_and_exports_every_declared_symbol():
    lib = cq.load()
    names = _declared()
    assert len(names) >= 9
    assert set(names) == set(cq.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert cq.cq_version() >= 100
    assert cq.status_string(cq.CQ_OK) == "CQ_OK"
    assert cq.status_string(cq.CQ_ERR_HIP) == "CQ_ERR_HIP"


@pytest.mark.parametrize("c,b", FORMATS)
def test_sizes_follow_bits_per_fpn_and_the_layout(c, b):
    fmt = cq.CQFormat(c, b, 128, 8)
    assert cq.cq_format_check(fmt) == cq.CQ_OK
    bpth = cq.cq_code_bytes_per_token_head(fmt)
    assert bpth * 8 == (128 // c) * b                     # dense: b / c bits per stored number
    assert bpth == L.bytes_per_token_head(c, b, 128)
    assert cq.cq_cache_bytes(fmt, 3, 256) == L.cache_bytes(c, b, 128, 8, 3, 256)
    assert cq.cq_cache_bytes(fmt, 3, 100) == 0            # t_cap must be a multiple of 64
    assert cq.cq_cache_bytes(fmt, 0, 128) == 0


def test_unsupported_and_invalid_formats():
    assert cq.cq_format_check(cq.CQFormat(3, 8, 128, 8)) == cq.CQ_ERR_INVALID_ARG     # 3 does not divide 128
    assert cq.cq_format_check(cq.CQFormat(0, 8, 128, 8)) == cq.CQ_ERR_INVALID_ARG
    assert cq.cq_format_check(cq.CQFormat(8, 9, 128, 8)) == cq.CQ_ERR_UNSUPPORTED
    assert cq.cq_format_check(cq.CQFormat(1, 8, 128, 8)) == cq.CQ_ERR_UNSUPPORTED
    assert cq.cq_format_check(cq.CQFormat(4, 10, 128, 8)) == cq.CQ_ERR_UNSUPPORTED
    assert cq.cq_code_bytes_per_token_head(cq.CQFormat(8, 9, 128, 8)) == 0
    assert int(cq.load().cq_format_check(None)) == cq.CQ_ERR_INVALID_ARG


def _fake(addr=0x10000):
    return ctypes.c_void_p(addr)


def _encode(fmt, x=0x10000, cen=0x20000, codes=0x30000, bstride=None, rstride=None, batch=1, t_new=64,
            t_offset=0, t_cap=64):
    f = fmt._c()
    rstride = fmt.channels if rstride is None else rstride
    bstride = rstride * t_new if bstride is None else bstride
    return int(cq.load().cq_encode(_fake(x), bstride, rstride, _fake(cen), ctypes.byref(f), batch, t_new,
                                   _fake(codes), t_offset, t_cap, None))


def test_encode_rejects_bad_arguments_without_launching():
    fmt = cq.CQFormat(8, 8, 128, 4)
    E = cq.CQ_ERR_INVALID_ARG
    assert _encode(fmt, x=0) == E
    assert _encode(fmt, cen=0) == E
    assert _encode(fmt, codes=0) == E
    assert _encode(fmt, x=0x10004) == E                    # misaligned
    assert _encode(fmt, batch=0) == E
    assert _encode(fmt, t_new=0) == E
    assert _encode(fmt, t_cap=100) == E
    assert _encode(fmt, t_offset=1, t_new=64, t_cap=64) == E
    assert _encode(fmt, t_offset=-1) == E
    assert _encode(fmt, rstride=fmt.channels - 8) == E
    assert _encode(fmt, rstride=fmt.channels + 4) == E     # rows would lose 16-byte alignment
    assert _encode(fmt, batch=2, bstride=8) == E
    assert _encode(cq.CQFormat(8, 9, 128, 4)) == cq.CQ_ERR_UNSUPPORTED


def _decode(fmt, batch=2, hq=8, t=128, t_cap=128, split=0, ws_bytes=1 << 30, ptrs=None, scale=0.1, seq=None):
    f = fmt._c()
    p = dict(q=0x10000, kc=0x20000, vc=0x30000, ck=0x40000, cv=0x50000, out=0x60000, ws=0x70000)
    p.update(ptrs or {})
    return int(cq.load().cq_decode_attention(_fake(p["q"]), _fake(p["kc"]), _fake(p["vc"]), _fake(p["ck"]),
                                             _fake(p["cv"]), scale, ctypes.byref(f), batch, hq, t, t_cap, seq,
                                             split, _fake(p["out"]), _fake(p["ws"]), ws_bytes, None))


def test_decode_rejects_bad_arguments_without_launching():
    fmt = cq.CQFormat(8, 8, 128, 4)
    E = cq.CQ_ERR_INVALID_ARG
    for k in ("q", "kc", "vc", "ck", "cv", "out", "ws"):
        assert _decode(fmt, ptrs={k: 0}) == E, k
    assert _decode(fmt, ptrs={"q": 0x10008}) == E
    assert _decode(fmt, hq=6) == E                         # not a multiple of the KV heads
    assert _decode(fmt, batch=0) == E
    assert _decode(fmt, t=0) == E
    assert _decode(fmt, t=129, t_cap=128) == E
    assert _decode(fmt, t_cap=96, t=64) == E
    assert _decode(fmt, split=100) == E                    # not a multiple of 64
    assert _decode(fmt, split=-64) == E
    assert _decode(cq.CQFormat(2, 8, 128, 4), split=64 * 129) == E      # beyond one chunk of scores (64 groups per head)
    assert _decode(cq.CQFormat(8, 10, 128, 4), split=64 * 257) == E     # ... (1024 centroids)
    assert _decode(fmt, scale=float("nan")) == E
    assert _decode(fmt, ws_bytes=16) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    assert _decode(cq.CQFormat(8, 7, 128, 4)) == cq.CQ_ERR_UNSUPPORTED


def _decode_static(fmt, batch=2, hq=8, t=128, t_cap=128, split=0, ptrs=None, scale=0.1):
    f = fmt._c()
    p = dict(q=0x10000, kc=0x20000, vc=0x30000, ck=0x40000, cv=0x50000, out=0x60000)
    p.update(ptrs or {})
    return int(cq.load().cq_decode_attention_static(_fake(p["q"]), _fake(p["kc"]), _fake(p["vc"]), _fake(p["ck"]),
                                                    _fake(p["cv"]), scale, ctypes.byref(f), batch, hq, t, t_cap, None,
                                                    split, _fake(p["out"]), None))


def test_static_scratch_decode_rejects_bad_arguments_and_sizes_without_launching():
    fmt = cq.CQFormat(8, 8, 128, 4)
    E = cq.CQ_ERR_INVALID_ARG
    for k in ("q", "kc", "vc", "ck", "cv", "out"):
        assert _decode_static(fmt, ptrs={k: 0}) == E, k
    assert _decode_static(fmt, hq=6) == E
    assert _decode_static(fmt, t=0) == E
    assert _decode_static(fmt, split=100) == E
    assert _decode_static(cq.CQFormat(8, 7, 128, 4)) == cq.CQ_ERR_UNSUPPORTED
    # partials beyond the 4 MiB array: 8066 rows of (2 + 128) floats do not fit, 8065 do (checked
    # through the size rule only: a fitting call would go on to launch)
    assert cq.STATIC_SCRATCH_BYTES == 4 << 20
    assert cq.STATIC_SCRATCH_BYTES // (130 * 4) == 8065
    big = cq.CQFormat(8, 8, 128, 32)
    assert _decode_static(big, batch=64, hq=32, t=4096, t_cap=4096, split=512) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    assert _decode_static(big, batch=1, hq=32, t=64 * 253, t_cap=64 * 253, split=64) == cq.CQ_ERR_WORKSPACE_TOO_SMALL


def test_workspace_size_matches_the_split_arithmetic():
    fmt = cq.CQFormat(8, 8, 128, 32)
    # explicit split: ceil(t / split) partials of (2 + head_dim) floats per (sequence, query head)
    assert cq.cq_decode_workspace_bytes(fmt, 4, 32, 1000, 256) == 4 * 32 * 4 * 130 * 4
    assert cq.cq_decode_workspace_bytes(fmt, 4, 32, 1024, 1024) == 4 * 32 * 1 * 130 * 4
    assert cq.cq_decode_workspace_bytes(fmt, 4, 32, 1000, 100) == 0
    d = cq.cq_decode_default_split(fmt, 4, 32, 131072)
    assert d % 64 == 0 and d > 0
    n_split = -(-131072 // d)
    assert cq.cq_decode_workspace_bytes(fmt, 4, 32, 131072, 0) == 4 * 32 * n_split * 130 * 4


def test_python_binding_refuses_cpu_tensors():
    import torch
    fmt = cq.CQFormat(8, 8, 128, 1)
    x = torch.zeros((1, 64, 128), dtype=torch.float16)
    cb = torch.zeros((16, 256, 8), dtype=torch.float16)
    codes = torch.zeros(1024, dtype=torch.uint8)
    with pytest.raises(TypeError):
        cq.cq_encode(x, cb, fmt, codes, 0, 64)


def test_probes_reject_bad_arguments_without_launching():
    lib = cq.load()
    assert lib.cq_probe_mfma(_fake(), _fake(0x20000), _fake(0x30000), 7, None) == cq.CQ_ERR_INVALID_ARG
    assert lib.cq_probe_mfma(None, _fake(0x20000), _fake(0x30000), 16, None) == cq.CQ_ERR_INVALID_ARG
    assert lib.cq_probe_mfma(_fake(0x10004), _fake(0x20000), _fake(0x30000), 8, None) == cq.CQ_ERR_INVALID_ARG
    assert lib.cq_probe_copy(_fake(), _fake(0x20000), 24, None) == cq.CQ_ERR_INVALID_ARG
    assert lib.cq_probe_stream_read(_fake(), 0, _fake(0x20000), None) == cq.CQ_ERR_INVALID_ARG


def test_kmeans_sizes_and_argument_checks_without_launching():
    lib = cq.load()
    f = cq.CQFormat(8, 8, 128, 2)._c()
    n = 1000
    G, K, c = 32, 256, 8
    need = lib.cq_kmeans_workspace_bytes(ctypes.byref(f), n)
    # tokens (group-major fp16), integer weights, nearest-centre distances, assignment, fp32 centroids, weight maxima
    assert need >= G * n * c * 2 + G * n * 4 + G * n * 4 + G * n * 2 + G * K * c * 4 + G * 4
    assert need < 1.02 * (G * n * c * 2 + G * n * 10 + G * K * c * 4) + 4096
    assert lib.cq_kmeans_workspace_bytes(ctypes.byref(f), 0) == 0
    assert lib.cq_kmeans_workspace_bytes(ctypes.byref(f), cq.KMEANS_MAX_POINTS + 1) == 0

    def fit(x=0x10000, stride=256, w=None, n_points=n, n_iter=3, rnd=0x20000, init=None, picks=None, cent=0x30000,
            cent32=None, assign=None, ws=0x40000, ws_bytes=need):
        p = lambda v: None if v is None else _fake(v)
        return int(lib.cq_kmeans_fit(p(x), stride, p(w), ctypes.byref(f), n_points, n_iter, p(rnd), p(init), p(picks),
                                     p(cent), p(cent32), p(assign), p(ws), ws_bytes, None))

    assert fit(x=None) == cq.CQ_ERR_INVALID_ARG
    assert fit(stride=255) == cq.CQ_ERR_INVALID_ARG and fit(stride=260) == cq.CQ_ERR_INVALID_ARG
    assert fit(n_points=0) == cq.CQ_ERR_INVALID_ARG and fit(n_iter=-1) == cq.CQ_ERR_INVALID_ARG
    assert fit(rnd=None) == cq.CQ_ERR_INVALID_ARG                    # no source of starting centroids
    assert fit(init=0x50000) == cq.CQ_ERR_INVALID_ARG                # two sources
    assert fit(rnd=None, init=0x50000, picks=0x60000) == cq.CQ_ERR_INVALID_ARG
    assert fit(cent=None) == cq.CQ_ERR_INVALID_ARG
    assert fit(x=0x10002) == cq.CQ_ERR_INVALID_ARG
    assert fit(ws=None) == cq.CQ_ERR_INVALID_ARG
    assert fit(ws_bytes=need - 1) == cq.CQ_ERR_WORKSPACE_TOO_SMALL


def test_dequantize_argument_checks_without_launching():
    lib = cq.load()
    f = cq.CQFormat(8, 8, 128, 2)._c()

    def deq(codes=0x10000, cen=0x20000, batch=2, t0=0, cnt=100, t_cap=128, out=0x30000, bs=100 * 256, rs=256):
        p = lambda v: None if v is None else _fake(v)
        return int(lib.cq_dequantize(p(codes), p(cen), ctypes.byref(f), batch, t0, cnt, t_cap, p(out), bs, rs, None))

    assert deq(codes=None) == cq.CQ_ERR_INVALID_ARG and deq(out=None) == cq.CQ_ERR_INVALID_ARG
    assert deq(t0=30, cnt=100) == cq.CQ_ERR_INVALID_ARG              # runs past t_cap
    assert deq(t_cap=100) == cq.CQ_ERR_INVALID_ARG
    assert deq(rs=255) == cq.CQ_ERR_INVALID_ARG and deq(rs=260) == cq.CQ_ERR_INVALID_ARG
    assert deq(bs=99 * 256) == cq.CQ_ERR_INVALID_ARG
    assert deq(out=0x30008) == cq.CQ_ERR_INVALID_ARG


def test_paged_argument_checks_without_launching():
    lib = cq.load()
    f = cq.CQFormat(8, 8, 128, 2)._c()
    assert lib.cq_paged_cache_bytes(ctypes.byref(f), 10) == 10 * 2 * 1024
    assert lib.cq_paged_cache_bytes(ctypes.byref(f), 0) == 0
    PT = cq._PageTable

    def dec(pt, t=100, ws_bytes=1 << 20):
        p = None if pt is None else ctypes.byref(pt)
        return int(lib.cq_decode_attention_paged(_fake(0x10000), _fake(0x20000), _fake(0x30000), _fake(0x40000),
                                                 _fake(0x50000), 0.1, ctypes.byref(f), 2, 4, t, p, None, 0,
                                                 _fake(0x60000), _fake(0x70000), ws_bytes, None))

    good = PT(8, 2, 2, 0x80000)
    assert dec(None) == cq.CQ_ERR_INVALID_ARG
    assert dec(PT(0, 2, 2, 0x80000)) == cq.CQ_ERR_INVALID_ARG            # no pages
    assert dec(PT(8, 2, 1, 0x80000)) == cq.CQ_ERR_INVALID_ARG            # row stride < max_tiles
    assert dec(PT(8, 2, 2, 0)) == cq.CQ_ERR_INVALID_ARG                  # no table
    assert dec(PT(8, 2, 2, 0x80002)) == cq.CQ_ERR_INVALID_ARG            # misaligned table
    assert dec(good, t=129) == cq.CQ_ERR_INVALID_ARG                     # beyond max_tiles * 64
    assert dec(good, ws_bytes=0) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    enc = int(lib.cq_encode_kv_paged(_fake(0x10000), _fake(0x20000), 256 * 100, 256, _fake(0x30000), _fake(0x40000),
                                     ctypes.byref(f), 2, 100, _fake(0x50000), _fake(0x60000), ctypes.byref(good), 30, None))
    assert enc == cq.CQ_ERR_INVALID_ARG                                  # 30 + 100 tokens > 128


def test_rope_sizes_and_argument_checks_without_launching():
    lib = cq.load()
    assert lib.cq_rope_table_bytes(128, 4096) == 8 * (64 * 64 + 64 * 64)      # 64 tiles + 64 lane offsets, 64 pairs each
    assert lib.cq_rope_table_bytes(128, 100) == 0 and lib.cq_rope_table_bytes(64, 4096) == 0
    assert lib.cq_rope_table_bytes(128, 0) == 0
    E = cq.CQ_ERR_INVALID_ARG
    tab = lambda base=1e4, hd=128, pos=4096, p=0x10000, nbytes=1 << 20: int(
        lib.cq_rope_table(base, hd, pos, _fake(p) if p else None, nbytes, None))
    assert tab(hd=64) == cq.CQ_ERR_UNSUPPORTED
    assert tab(pos=100) == E and tab(pos=0) == E and tab(p=0) == E and tab(p=0x10004) == E
    assert tab(base=1.0) == E and tab(base=float("nan")) == E and tab(base=float("inf")) == E
    assert tab(nbytes=1024) == cq.CQ_ERR_WORKSPACE_TOO_SMALL

    def dec(fmt, t=128, t_cap=128, split=0, table=0x80000, positions=4096, ws_bytes=1 << 30):
        f = fmt._c()
        return int(lib.cq_decode_attention_rope(_fake(0x10000), _fake(0x20000), _fake(0x30000), _fake(0x40000),
                                                _fake(0x50000), 0.1, ctypes.byref(f), 2, 8, t, t_cap, None, split,
                                                _fake(table) if table else None, positions, _fake(0x60000),
                                                _fake(0x70000), ws_bytes, None))
    fmt = cq.CQFormat(4, 8, 128, 4)
    assert dec(fmt, table=0) == E and dec(fmt, table=0x80004) == E
    assert dec(fmt, positions=0) == E and dec(fmt, positions=100) == E
    assert dec(fmt, t=128, t_cap=128, positions=64) == E           # table shorter than the context
    assert dec(fmt, split=64 * 257, t=64 * 300, t_cap=64 * 300, positions=64 * 300) == E   # beyond the score buffer
    assert dec(fmt, ws_bytes=16) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    assert dec(cq.CQFormat(2, 4, 128, 4)) == cq.CQ_ERR_UNSUPPORTED     # sub-byte: through the fused format
    assert cq.cq_decode_rope_default_split(cq.CQFormat(8, 10, 128, 4), 2, 8, 4096) > 0
    f64 = cq.CQFormat(8, 8, 64, 4)._c()                                 # head_dim 128 only
    assert lib.cq_decode_step_rope(_fake(0x10000), _fake(0x11000), _fake(0x12000), 256, _fake(0x20000), _fake(0x30000),
                                   _fake(0x40000), _fake(0x50000), 0.1, ctypes.byref(f64), 2, 8, 128, 128, None, 0,
                                   _fake(0x80000), 4096, _fake(0x60000), _fake(0x70000), 1 << 30, None) == cq.CQ_ERR_UNSUPPORTED
    # several query tokens over such caches.  One or two tokens (library's split): the workspace of the
    # largest of the m single-token calls; more, or a split of the caller's: that of the matrix-core kernel
    assert cq.cq_chunk_rope_workspace_bytes(fmt, 2, 8, 2, 4096) == max(
        cq.cq_decode_workspace_bytes(fmt, 2, 8, t, cq.cq_decode_rope_default_split(fmt, 2, 8, t)) for t in (4095, 4096))
    assert cq.cq_chunk_rope_workspace_bytes(fmt, 2, 8, 3, 4096) == 4 * 2 * 3 * 8 * 130 * (4096 // cq.cq_chunk_default_split(fmt, 2, 8, 3, 4096))
    assert cq.cq_chunk_rope_workspace_bytes(fmt, 2, 8, 2, 4096, 1024) == 4 * 2 * 2 * 8 * 4 * 130
    assert cq.cq_chunk_rope_workspace_bytes(fmt, 2, 8, 5000, 4096) == 0 and cq.cq_chunk_rope_workspace_bytes(fmt, 2, 8, 3, 4096, 100) == 0

    def chunk(m=3, t=128, t_cap=128, ws_bytes=1 << 30, pos=4096, split=0, table=0x80000):
        return int(lib.cq_chunk_attention_rope(_fake(0x10000), _fake(0x20000), _fake(0x30000), _fake(0x40000), _fake(0x50000),
                                               0.1, ctypes.byref(fmt._c()), 2, 8, m, t, t_cap, None, split, _fake(table) if table else None, pos,
                                               _fake(0x60000), _fake(0x70000), ws_bytes, None))
    assert chunk(m=0) == cq.CQ_ERR_INVALID_ARG and chunk(m=129) == cq.CQ_ERR_INVALID_ARG and chunk(pos=0) == cq.CQ_ERR_INVALID_ARG
    assert chunk(split=100) == cq.CQ_ERR_INVALID_ARG and chunk(m=2, ws_bytes=16) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    # the matrix-core form: table and workspace checks
    assert chunk(t=4096, t_cap=4096, split=64, ws_bytes=16) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    assert chunk(t=4096, t_cap=4096, split=64, table=0) == cq.CQ_ERR_INVALID_ARG
    assert chunk(t=4096, t_cap=4096, split=64, table=0x80004) == cq.CQ_ERR_INVALID_ARG
    assert chunk(t=4096, t_cap=4096, split=64, pos=2048) == cq.CQ_ERR_INVALID_ARG      # table shorter than the context
    assert chunk(t=4096, t_cap=4096, split=64, pos=4100) == cq.CQ_ERR_INVALID_ARG
    assert cq.cq_decode_rope_default_split(cq.CQFormat(2, 8, 128, 32), 64, 32, 64 * 1000) == 64 * 250    # 4 balanced splits of at most 256 tiles


def test_layer_table_argument_checks_without_copying():
    lib = cq.load()
    assert lib.cq_layer_table_bytes(32) == 32 * 8 * 8 and lib.cq_layer_table_bytes(0) == 0
    E = cq.CQ_ERR_INVALID_ARG

    def rec(n=2, **kw):
        r = (cq._LayerIO * n)()
        for i in range(n):
            for j, name in enumerate(cq.LayerTable.FIELDS):
                setattr(r[i], name, 0x100000 * (i + 1) + 0x1000 * (j + 1))
        for k, v in kw.items():
            setattr(r[n - 1], k, v)
        return r
    fill = lambda r, n=2, table=0x900000, nbytes=1 << 12: int(lib.cq_layer_table_fill(r, n, _fake(table) if table else None, nbytes, None))
    assert fill(None) == E and fill(rec(), n=0) == E and fill(rec(), table=0) == E and fill(rec(), table=0x900008) == E
    assert fill(rec(), nbytes=64) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    for name in cq.LayerTable.FIELDS:
        assert fill(rec(**{name: 0})) == E, name
        assert fill(rec(**{name: 0x555554})) == E, name
    assert fill(rec(v_codes=0x200000 + 0x4000)) == E          # a layer's K and V caches coincide
    assert fill(rec(k_codes=0x100000 + 0x4000)) == E          # two layers share a cache
    assert fill(rec(out=0x100000 + 0x8000)) == E              # two layers share an output
    f = cq.CQFormat(4, 8, 128, 4)._c()
    step = lambda table=0x900000, n=2, stride=512, ws=1 << 30: int(lib.cq_decode_step_layers(
        _fake(table) if table else None, n, stride, 0.1, ctypes.byref(f), 2, 8, 128, 128, None, 0, _fake(0x70000), ws, None))
    assert step(table=0) == E and step(n=0) == E and step(stride=100) == E and step(table=0x900004) == E
    assert step(ws=cq.cq_decode_workspace_bytes(cq.CQFormat(4, 8, 128, 4), 2, 8, 128)) == cq.CQ_ERR_WORKSPACE_TOO_SMALL   # one layer's worth


def test_chunk_attention_sizes_and_argument_checks_without_launching():
    lib = cq.load()
    fmt = cq.CQFormat(4, 8, 128, 4)
    f = fmt._c()
    E = cq.CQ_ERR_INVALID_ARG
    # batch 16 x 4 KV heads x 1 row block = 64 workgroups: the context of 64 tiles is cut in 8
    assert cq.cq_chunk_default_split(fmt, 16, 8, 16, 4096) == 512
    assert cq.cq_chunk_workspace_bytes(fmt, 16, 8, 16, 4096) == 4 * 16 * 16 * 8 * 8 * 130
    # plenty of rows: one split
    assert cq.cq_chunk_default_split(fmt, 64, 32, 512, 4096) == 4096
    assert cq.cq_chunk_default_split(cq.CQFormat(8, 10, 128, 4), 16, 8, 16, 4096) == 512
    assert cq.cq_chunk_default_split(cq.CQFormat(2, 4, 128, 4), 16, 8, 16, 4096) == 0        # sub-byte: through the fused format
    assert cq.cq_chunk_default_split(fmt, 16, 8, 5000, 4096) == 0            # more queries than cached tokens
    # chunks of one or two tokens (up to 8 with one query head per KV head on large batches) are
    # served token by token by the single-token kernel: its split, its workspace
    assert cq.cq_chunk_default_split(fmt, 16, 8, 2, 4096) == cq.cq_decode_default_split(fmt, 16, 8, 4096)
    assert cq.cq_chunk_workspace_bytes(fmt, 1, 8, 2, 65536) == max(cq.cq_decode_workspace_bytes(fmt, 1, 8, t) for t in (65535, 65536))
    assert cq.cq_chunk_workspace_bytes(fmt, 1, 8, 2, 65536) > 0
    assert cq.cq_chunk_workspace_bytes(fmt, 16, 8, 2, 4096) == cq.cq_decode_workspace_bytes(fmt, 16, 8, 4096)
    mha = cq.CQFormat(4, 8, 128, 32)
    assert cq.cq_chunk_default_split(mha, 16, 32, 8, 4096) == cq.cq_decode_default_split(mha, 16, 32, 4096)
    assert cq.cq_chunk_workspace_bytes(mha, 16, 32, 8, 4096) == 0             # one split per token: nothing to merge
    assert cq.cq_chunk_workspace_bytes(mha, 16, 32, 9, 4096) == 4 * 16 * 9 * 32 * (4096 // cq.cq_chunk_default_split(mha, 16, 32, 9, 4096)) * 130

    def run(fm=f, q=0x10000, m=16, t=128, t_cap=128, split=0, ws=0x70000, ws_bytes=1 << 30, hq=8, scale=0.1):
        return int(lib.cq_chunk_attention(_fake(q) if q else None, _fake(0x20000), _fake(0x30000), _fake(0x40000),
                                          _fake(0x50000), scale, ctypes.byref(fm), 2, hq, m, t, t_cap, None, split,
                                          _fake(0x60000), _fake(ws) if ws else None, ws_bytes, None))
    assert run(q=0) == E and run(q=0x10004) == E and run(m=0) == E and run(m=129) == E and run(t=129) == E
    assert run(t_cap=100) == E and run(split=100) == E and run(hq=6) == E and run(scale=float("inf")) == E
    assert run(split=64, ws=0) == E                                          # split context needs the workspace
    assert run(split=64, ws_bytes=64) == cq.CQ_ERR_WORKSPACE_TOO_SMALL
    assert run(fm=cq.CQFormat(2, 4, 128, 4)._c()) == cq.CQ_ERR_UNSUPPORTED


def test_subbyte_formats_sizes_and_argument_checks_without_launching():
    lib = cq.load()
    for (c, b), (cf, bytes_th) in {(1, 2): (4, 32), (2, 2): (8, 16), (1, 4): (2, 64), (2, 4): (4, 32), (4, 4): (8, 16)}.items():
        fmt = cq.CQFormat(c, b, 128, 4)
        fused = cq.cq_fused_format(fmt)
        assert (fused.c, fused.b) == (cf, 8)
        assert cq.cq_code_bytes_per_token_head(fmt) == bytes_th == 128 * b // c // 8
    assert cq.cq_fused_format(cq.CQFormat(8, 10, 128, 4)) == cq.CQFormat(8, 10, 128, 4)
    f = cq.CQFormat(2, 4, 128, 4)._c()
    E = cq.CQ_ERR_INVALID_ARG
    assert lib.cq_expand_codebook(None, ctypes.byref(f), _fake(0x20000), None) == E
    assert lib.cq_expand_codebook(_fake(0x10000), ctypes.byref(f), _fake(0x10000), None) == E
    assert lib.cq_expand_codebook(_fake(0x10004), ctypes.byref(f), _fake(0x20000), None) == E
    f8 = cq.CQFormat(4, 8, 128, 4)._c()
    assert lib.cq_expand_codebook(_fake(0x10000), ctypes.byref(f8), _fake(0x20000), None) == E
    assert lib.cq_fused_format(ctypes.byref(f), None) == E
    bad = cq.CQFormat(8, 4, 128, 4)._c()
    assert lib.cq_fused_format(ctypes.byref(bad), ctypes.byref(f8)) == cq.CQ_ERR_UNSUPPORTED
    # the decode side refuses the sub-byte format itself
    assert _decode(cq.CQFormat(2, 4, 128, 4)) == cq.CQ_ERR_UNSUPPORTED


def test_default_split_is_balanced_within_the_on_chip_limits_and_fills_the_chip():
    import numpy as np
    rng = np.random.default_rng(11)
    limit = {(8, 8): 1 << 26, (4, 8): 1 << 26, (2, 8): 8192, (8, 10): 16384}
    for _ in range(300):
        c, b = [(8, 8), (4, 8), (2, 8), (8, 10)][int(rng.integers(0, 4))]
        hkv = int(rng.choice([1, 2, 8, 32]))
        hq = hkv * int(rng.choice([1, 4]))
        B = int(rng.choice([1, 2, 16, 64]))
        T = int(rng.integers(1, 200000))
        fmt = cq.CQFormat(c, b, 128, hkv)
        split = cq.cq_decode_default_split(fmt, B, hq, T)
        assert split > 0 and split % 64 == 0 and split <= limit[(c, b)]
        tiles, n_tiles = split // 64, -(-T // 64)
        n_split = -(-n_tiles // tiles)
        assert tiles == -(-n_tiles // n_split)                     # equal splits: no short last one beyond rounding
        assert n_split == 1 or tiles >= 16 or n_tiles < 32         # never shorter than 16 tiles by choice
        assert cq.cq_decode_workspace_bytes(fmt, B, hq, T) == 4 * B * hq * n_split * 130
    # the named workloads
    assert cq.cq_decode_default_split(cq.CQFormat(4, 8, 128, 32), 16, 32, 4096) == 4096        # one split, no merge
    assert cq.cq_decode_default_split(cq.CQFormat(8, 8, 128, 32), 4, 32, 131072) == 32768      # 4 x 512 tiles: all 512 workgroups at once
    assert cq.cq_decode_default_split(cq.CQFormat(8, 10, 128, 8), 32, 32, 16384) == 16384
    assert cq.cq_decode_default_split(cq.CQFormat(8, 8, 128, 32), 1, 32, 131072) == 16384      # shorter job: one workgroup per CU
    assert cq.cq_decode_default_split(cq.CQFormat(8, 8, 128, 32), 8, 32, 16384) == 16384       # 256 rows: no split at all
    assert cq.cq_decode_default_split(cq.CQFormat(4, 8, 128, 32), 1, 32, 32768) == 4096
