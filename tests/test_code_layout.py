"""Pins for the packed-cache layout as restated in numpy (oracle/code_layout.py) and for
the shape bookkeeping of the paper: densities of Table 1, codebook sizes of Table 5.
CPU only."""
import os

import numpy as np
import pytest

import synth
from oracle import code_layout as L

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_bits_per_fpn_match_table_1():
    for name, c, b, printed in _rows("table1_bits_per_fpn.txt"):
        assert L.bits_per_fpn(int(c), int(b), 128) == pytest.approx(float(printed), abs=0.005), name
        # the packed record really has that many bytes: no padding
        assert L.bytes_per_token_head(int(c), int(b), 128) * 8 == (128 // int(c)) * int(b)


def test_codebook_sizes_match_table_5():
    # a codebook tensor [G, 2^b, c] per layer and per K/V, G = kv_heads * head_dim / c
    for model, layers, hkv, hd, b, printed in _rows("table5_centroid_params.txt"):
        layers, hkv, hd, b = int(layers), int(hkv), int(hd), int(b)
        for c in (2, 4, 8):
            G = hkv * hd // c
            count = layers * 2 * G * (1 << b) * c
            assert count == layers * 2 * hkv * hd * (1 << b)
            assert round(count / 1e6, 2) == pytest.approx(float(printed), abs=0.006), model
    # the synthetic codebooks have exactly that shape
    r = synth.tensor_recipe(1, 0, "k", 4096)
    for c in (2, 4, 8):
        assert synth.sample_codebook(r, c, 8).shape == (4096 // c, 256, c)
        assert synth.sample_codebook(r, c, 8).size == 32 * 128 * 256


def test_16x_compression_at_one_bit_per_channel():
    # abstract / introduction: 1 bit per fp16 number is 16x compression
    fp16_bytes = 128 * 2
    assert fp16_bytes / L.bytes_per_token_head(8, 8, 128) == 16


@pytest.mark.parametrize("c,b,hkv", [(8, 8, 3), (4, 8, 2), (2, 8, 2), (8, 10, 2)])
def test_pack_unpack_round_trip(c, b, hkv):
    rng = np.random.default_rng(c * 100 + b)
    B, T, t_cap, t_off = 2, 150, 256, 37
    G = hkv * 128 // c
    codes = rng.integers(0, 1 << b, size=(B, T, G)).astype(np.uint16)
    codes[0, 0, :] = 0
    codes[0, 1, :] = (1 << b) - 1
    cache = L.pack(codes, c, b, 128, hkv, t_cap, t_offset=t_off, fill=0xA5)
    assert cache.dtype == np.uint8
    assert cache.size == L.cache_bytes(c, b, 128, hkv, B, t_cap)
    assert np.array_equal(L.unpack(cache, c, b, 128, hkv, T, t_off), codes)
    # tokens outside [t_off, t_off+T) are untouched
    before = L.unpack(np.full_like(cache, 0xA5), c, b, 128, hkv, t_off, 0)
    assert np.array_equal(L.unpack(cache, c, b, 128, hkv, t_off, 0), before)
    # incremental append equals one-shot packing
    cache2 = L.pack(codes[:, :100], c, b, 128, hkv, t_cap, t_offset=t_off, fill=0xA5)
    L.pack(codes[:, 100:], c, b, 128, hkv, t_cap, t_offset=t_off + 100, into=cache2)
    assert np.array_equal(cache2, cache)


def test_byte_positions_written_out_by_hand_8bit():
    # CQ-8c8b, one head (16 groups), token t = 67 (tile 1, u = 3), group g = 5:
    # slot s = (g - u) mod 16 = 2 -> plane 0, byte 3*16 + 2 of tile 1.
    codes = np.zeros((1, 128, 16), dtype=np.uint16)
    codes[0, 67, 5] = 0xC7
    cache = L.pack(codes, 8, 8, 128, 1, 128)
    flat = cache.reshape(-1)
    assert flat[1 * 1024 + 3 * 16 + 2] == 0xC7 and np.count_nonzero(flat) == 1
    # CQ-2c8b, two heads (64 groups each), sequence 0, head 1, t = 70 (tile 1, u = 6), group 3:
    # slot s = (3 - 6) mod 64 = 61 -> plane 3, byte 13; stream of head 1 starts after head 0's 2 tiles.
    codes = np.zeros((1, 128, 128), dtype=np.uint16)
    codes[0, 70, 64 + 3] = 0x11
    cache = L.pack(codes, 2, 8, 128, 2, 128)
    flat = cache.reshape(-1)
    tile = 64 * 64
    assert flat[2 * tile + 1 * tile + 3 * 1024 + 6 * 16 + 13] == 0x11 and np.count_nonzero(flat) == 1


def test_byte_positions_written_out_by_hand_10bit():
    # CQ-8c10b, token u = 2 of tile 0, group 7 -> slot 5; code 0x2B4 = high bits 0b10, low byte 0xB4.
    codes = np.zeros((1, 64, 16), dtype=np.uint16)
    codes[0, 2, 7] = 0x2B4
    cache = L.pack(codes, 8, 10, 128, 1, 64)
    flat = cache.reshape(-1)
    assert flat.size == 64 * 20
    assert flat[2 * 16 + 5] == 0xB4
    word = int.from_bytes(bytes(flat[1024 + 2 * 4:1024 + 2 * 4 + 4]), "little")
    assert word == (0b10 << 10)
    assert np.count_nonzero(flat) == 2


def test_in_each_slot_the_64_tokens_of_a_tile_cover_the_groups_evenly():
    # the rotation puts, in any fixed slot, 64/Gh tokens on every group
    for c in (8, 4, 2):
        Gh = 128 // c
        codes = np.tile(np.arange(Gh, dtype=np.uint16), (1, 64, 1))      # code == group id
        cache = L.pack(codes, c, 8, 128, 1, 64).reshape(Gh // 16, 64, 16)
        for p in range(Gh // 16):
            for w in range(16):
                assert np.array_equal(np.bincount(cache[p, :, w], minlength=Gh), np.full(Gh, 64 // Gh))
                assert np.array_equal(cache[p, :, w], (16 * p + w + np.arange(64)) % Gh)


def test_rejects_bad_shapes():
    codes = np.zeros((1, 10, 16), dtype=np.uint16)
    with pytest.raises(ValueError):
        L.pack(codes, 8, 8, 128, 1, 100)                 # t_cap not a multiple of 64
    with pytest.raises(ValueError):
        L.pack(codes, 8, 8, 128, 1, 64, t_offset=60)     # does not fit
    with pytest.raises(ValueError):
        L.pack(codes + 256, 8, 8, 128, 1, 64)            # code out of range
    with pytest.raises(ValueError):
        L.pack(codes, 8, 9, 128, 1, 64)
