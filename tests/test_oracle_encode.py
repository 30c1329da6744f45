"""Pins for the oracle's encoder (Section 3.2 of the paper: nearest centroid in L2 per
group of c contiguous channels), against things other than the oracle itself:
pure-Python brute force, library vector quantizers, closed-form special cases and
tie-break constructions.  CPU only."""
import numpy as np
import pytest

from oracle import cq_oracle as O


def _rand_case(seed, T, G, K, c, scale=1.0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((T, G * c)) * scale).astype(np.float16)
    cb = (rng.standard_normal((G, K, c)) * scale).astype(np.float16)
    return x, cb


def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_to_double(int(v)) for v in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    # signed zeros keep their sign
    assert np.signbit(O.half_to_double(0x8000)) and not np.signbit(O.half_to_double(0x0000))


@pytest.mark.parametrize("c,b", [(1, 2), (2, 4), (3, 3), (4, 8), (8, 8), (8, 10)])
def test_encode_equals_pure_python_brute_force(c, b):
    T, G, K = 5, 3, 1 << b
    x, cb = _rand_case(100 + c * 16 + b, T, G, K, c)
    codes = O.encode(x, cb)
    for t in range(T):
        for g in range(G):
            best_j, best_d = None, None
            for j in range(K):
                d = 0.0
                for i in range(c):
                    diff = float(x[t, g * c + i]) - float(cb[g, j, i])
                    d += diff * diff
                if best_d is None or d < best_d:
                    best_j, best_d = j, d
            assert codes[t, g] == best_j


def test_encode_equals_scipy_vq_per_group():
    from scipy.cluster.vq import vq
    c, b, T, G = 4, 8, 200, 6
    x, cb = _rand_case(7, T, G, 1 << b, c)
    codes, d1, _ = O.encode(x, cb, with_distances=True)
    for g in range(G):
        obs = x[:, g * c:(g + 1) * c].astype(np.float64)
        lib_codes, lib_dist = vq(obs, cb[g].astype(np.float64))
        assert np.array_equal(codes[:, g], lib_codes)
        np.testing.assert_allclose(np.sqrt(d1[:, g]), lib_dist, rtol=1e-12, atol=1e-300)


def test_encode_equals_torch_cdist_argmin():
    import torch
    c, b, T, G = 8, 8, 128, 4
    x, cb = _rand_case(11, T, G, 1 << b, c, scale=3.0)
    codes = O.encode(x, cb)
    for g in range(G):
        xs = torch.from_numpy(x[:, g * c:(g + 1) * c].astype(np.float64))
        cs = torch.from_numpy(cb[g].astype(np.float64))
        want = torch.cdist(xs, cs, compute_mode="donot_use_mm_for_euclid_dist").argmin(dim=1).numpy()
        assert np.array_equal(codes[:, g], want)


def test_encode_is_optimal_and_reports_two_smallest_distances():
    c, b, T, G = 2, 8, 64, 8
    x, cb = _rand_case(13, T, G, 1 << b, c)
    codes, d1, d2 = O.encode(x, cb, with_distances=True)
    xg = x.astype(np.float64).reshape(T, G, 1, c)
    dist = ((xg - cb.astype(np.float64)[None]) ** 2).sum(-1)          # [T, G, K]
    part = np.sort(dist, axis=-1)
    np.testing.assert_allclose(d1, part[..., 0], rtol=1e-13)
    np.testing.assert_allclose(d2, part[..., 1], rtol=1e-13)
    chosen = np.take_along_axis(dist, codes[..., None].astype(np.int64), axis=-1)[..., 0]
    assert np.all(chosen <= dist.min(-1) * (1 + 1e-15))


def test_groups_are_contiguous_channel_slices_with_their_own_codebooks():
    # group g must read channels [g c, g c + c) and codebook g only: build a codebook whose
    # entry j of group g equals token j's slice of group g, so token t must get code t everywhere.
    c, G, K = 4, 5, 16
    rng = np.random.default_rng(3)
    x = rng.standard_normal((K, G * c)).astype(np.float16)
    cb = np.ascontiguousarray(x.reshape(K, G, c).transpose(1, 0, 2))
    codes, d1, _ = O.encode(x, cb, with_distances=True)
    assert np.array_equal(codes, np.repeat(np.arange(K)[:, None], G, axis=1))
    assert np.all(d1 == 0.0)
    # a codebook permuted across groups no longer reproduces it
    codes2 = O.encode(x, np.roll(cb, 1, axis=0))
    assert not np.array_equal(codes2, codes)


def test_ties_go_to_lowest_index():
    c, K = 2, 8
    # (a) all centroids identical -> every code is 0
    cb = np.tile(np.array([[0.5, -1.0]], dtype=np.float16), (1, K, 1))
    x = np.random.default_rng(0).standard_normal((10, c)).astype(np.float16)
    assert np.all(O.encode(x, cb) == 0)
    # (b) a duplicate of a centroid at a higher index is never emitted
    rng = np.random.default_rng(1)
    cb = rng.standard_normal((1, K, c)).astype(np.float16)
    cb[0, 6] = cb[0, 2]
    x = rng.standard_normal((500, c)).astype(np.float16)
    codes = O.encode(x, cb)
    assert 2 in codes and 6 not in codes
    # (c) x exactly midway between two centroids -> the lower index
    cb = np.array([[[10, 10], [1.0, 0.0], [-1.0, 0.0], [10, -10]]], dtype=np.float16)
    x = np.array([[0.0, 0.25]], dtype=np.float16)
    codes, d1, d2 = O.encode(x, cb, with_distances=True)
    assert codes[0, 0] == 1 and d1[0, 0] == d2[0, 0]
    cb2 = cb[:, [0, 2, 1, 3]]
    assert O.encode(x, cb2)[0, 0] == 1


def test_c1_with_every_input_value_in_the_codebook_reconstructs_exactly():
    # c = 1 is non-uniform channel-wise quantization (Eq. 2, Section 2.3).
    rng = np.random.default_rng(5)
    D, K, T = 6, 32, 300
    levels = rng.standard_normal((D, K)).astype(np.float16)
    pick = rng.integers(0, K, size=(T, D))
    x = levels[np.arange(D)[None, :], pick]
    cb = levels.reshape(D, K, 1)
    codes = O.encode(x, cb)
    recon = O.dequantize(codes, cb)
    assert np.array_equal(recon, x.astype(np.float64))
    # and it is the textbook scalar nearest-level rule on arbitrary inputs
    x2 = rng.standard_normal((T, D)).astype(np.float16)
    codes2 = O.encode(x2, cb)
    want = np.abs(x2.astype(np.float64)[:, :, None] - levels.astype(np.float64)[None]).argmin(-1)
    assert np.array_equal(codes2, want)


def test_encode_of_dequantized_codes_is_the_identity_when_centroids_are_distinct():
    c, b, G, T = 4, 8, 3, 400
    rng = np.random.default_rng(9)
    cb = rng.standard_normal((G, 1 << b, c)).astype(np.float16)
    codes = rng.integers(0, 1 << b, size=(T, G)).astype(np.uint16)
    recon = O.dequantize(codes, cb)
    # dequantize is a plain table lookup
    want = np.stack([cb[g, codes[:, g]] for g in range(G)], axis=1).reshape(T, G * c)
    assert np.array_equal(recon, want.astype(np.float64))
    again = O.encode(recon.astype(np.float16), cb)
    assert np.array_equal(again, codes)


def test_quantization_error_is_the_sum_of_best_distances():
    # || A - CQ(A) ||_F^2 of Eq. 5 equals the sum of the per-(token, group) minima.
    c, b, G, T = 8, 8, 4, 50
    x, cb = _rand_case(21, T, G, 1 << b, c)
    codes, d1, _ = O.encode(x, cb, with_distances=True)
    err = ((x.astype(np.float64) - O.dequantize(codes, cb)) ** 2).sum()
    np.testing.assert_allclose(err, d1.sum(), rtol=1e-12)


def test_bad_arguments_are_rejected():
    x, cb = _rand_case(1, 4, 2, 4, 2)
    with pytest.raises(ValueError):
        O.encode(x[:, :3], cb)
    with pytest.raises(TypeError):
        O.encode(x.astype(np.float32), cb)
