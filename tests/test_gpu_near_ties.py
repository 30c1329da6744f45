"""Nearest-centroid search AT the acceptance boundary (Section 3.2: "nearest centroid in terms of L2
distance"; ties and near-ties are this build's reading): tokens are planted whose two nearest
centroids differ by a TRUE relative gap (d2 - d1) / d2, measured by the fp64 oracle, inside
[1e-6, 3e-6] -- there the library must return the oracle's code bit for bit -- and inside
[1e-8, 1e-6) -- there it may pick either of the two, never anything else.  The nearer centroid
always sits at the HIGHER index, so a search that cannot tell the two apart (and falls back to the
lowest index) is caught.  Every encode path: the matrix-core kernel (many tokens), the
lane-per-centroid kernel (a handful), the fused decode step (one new token per sequence).

Why the first band must be exact: the kernels decide close calls with the direct fp32 form
(rounded difference, one fused multiply-add per channel, channel order).  Where the differences
are exact in fp32, the c fused multiply-adds err by at most c 2^-24 of the sum, so two
distances compare correctly when they differ by more than 2 c 2^-24 = 9.6e-7 (c = 8) of
themselves.  The planted differences are exact: channel 0 holds -0.5 / +0.5 against a small
token value (every fp16 number is a multiple of 2^-24, the difference is below 1: 24 bits), the
other channels hold numbers of magnitude 0.25 to 4 (multiples of 2^-12, differences below 8)."""
import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
from oracle import cq_oracle as O

from gpu_util import cache_to_codes, check_codes, codes_to_cache, dev, gpu_encode

pytestmark = pytest.mark.gpu

BAND_EXACT = (1.0e-6, 3.0e-6)
BAND_LOOSE = (1.0e-8, 1.0e-6)


def _plant(c, b, n_groups, n_tokens, band, seed):
    """Codebook fp16 [G, 2^b, c] and tokens fp16 [n_tokens, G c]: in every group, centroid j_hi is
    the nearest of every token and centroid j_lo < j_hi the runner-up, with a relative gap of the
    squared fp64 distances inside `band`; all other centroids are far away.

    The two centroids are -0.5 and +0.5 in channel 0 and arbitrary elsewhere.  A token starts on
    their bisector plane with channel 0 at zero; rounding its other channels to fp16 leaves a gap
    of about +-1e-3, which channel 0 (a number of magnitude 1e-4, where fp16 is spaced 1e-7 apart)
    then moves to a target drawn inside the band."""
    rng = np.random.default_rng(seed)
    K = 1 << b
    cb = np.empty((n_groups, K, c), dtype=np.float16)
    x = np.empty((n_tokens, n_groups, c), dtype=np.float16)
    lo_t, hi_t = band[0] + 0.15 * (band[1] - band[0]), band[1] - 0.15 * (band[1] - band[0])
    for g in range(n_groups):
        j_lo, j_hi = sorted(rng.choice(K, size=2, replace=False))
        # the two centroids: midpoint and half difference on a grid of 2^-7, so that the midpoint is an
        # fp16 number as well
        mid = np.round(rng.uniform(0.5, 2.0, size=c) * rng.choice([-1.0, 1.0], size=c) * 128) / 128
        half = np.round(rng.uniform(0.125, 0.5, size=c) * rng.choice([-1.0, 1.0], size=c) * 128) / 128
        mid[0], half[0] = 0.0, 0.5
        near, far = mid - half, mid + half
        near16, far16 = near.astype(np.float16), far.astype(np.float16)
        assert np.array_equal(near16.astype(np.float64), near) and np.array_equal(far16.astype(np.float64), far)
        # everything else: well away from the segment between the two
        others = (near + rng.uniform(4.0, 8.0, size=(K, c)) * rng.choice([-1.0, 1.0], size=(K, c))).astype(np.float16)
        cb[g] = others
        cb[g, j_hi], cb[g, j_lo] = near16, far16
        a, f = near16.astype(np.float64), far16.astype(np.float64)
        mid, rest = 0.5 * (a + f), f - a
        rest[0] = 0.0                       # (channel 0 of the bisector's midpoint is 0: it drops out at x0 = 0)
        got = np.empty((0, c), dtype=np.float16)
        for _ in range(200):
            if len(got) >= n_tokens:
                break
            cand = mid + rng.normal(0.0, 0.15, size=(4 * n_tokens, c))
            cand[:, 0] = 0.0
            cand -= np.outer((cand - mid) @ rest / (rest @ rest), rest)
            c64 = cand.astype(np.float16).astype(np.float64)
            d_far = ((c64 - f) ** 2).sum(-1)
            g0 = (d_far - ((c64 - a) ** 2).sum(-1)) / d_far
            target = rng.uniform(lo_t, hi_t, size=len(c64))
            c64[:, 0] = ((g0 - target) * d_far / 2.0).astype(np.float16).astype(np.float64)     # d gap / d x0 = -2 / d_far
            d_far = ((c64 - f) ** 2).sum(-1)
            gap = (d_far - ((c64 - a) ** 2).sum(-1)) / d_far
            # (channel 0 below 2^-12: there fp16 numbers are at most 1.2e-7 apart)
            ok = (gap >= band[0]) & (gap < band[1]) & (np.abs(c64[:, 0]) < 2.0 ** -12)
            got = np.concatenate([got, c64[ok].astype(np.float16)])
        assert len(got) >= n_tokens, "planting failed"
        x[:, g] = got[:n_tokens]
    return cb, x.reshape(n_tokens, n_groups * c)


def _check_planted(x, cb, band):
    ref, d1, d2 = O.encode(x, cb, with_distances=True)
    gap = (d2 - d1) / d2
    assert gap.min() >= band[0] and gap.max() < band[1], (gap.min(), gap.max())
    return ref


@pytest.mark.parametrize("c", [2, 4, 8])
@pytest.mark.parametrize("band", [BAND_EXACT, BAND_LOOSE], ids=["gap_1e-6_to_3e-6", "gap_1e-8_to_1e-6"])
def test_prefill_and_small_encode_at_the_boundary(c, band):
    b, hkv = 8, 1
    fmt = cq.CQFormat(c, b, 128, hkv)
    cb, x = _plant(c, b, fmt.groups, 320, band, 1000 * c + int(band[0] * 1e9))
    ref = _check_planted(x, cb, band)
    # the matrix-core kernel: one sequence of 320 tokens (five tiles); the lane-per-centroid
    # kernel: 20 sequences of 16 tokens
    for shape in ((1, 320), (20, 16)):
        B, T = shape
        t_cap = (T + 63) // 64 * 64
        cache = gpu_encode(x.reshape(B, T, -1), cb, fmt, t_cap)
        got = cache_to_codes(cache, fmt, B, t_cap, T).reshape(B * T, -1)
        if band is BAND_EXACT:
            assert np.array_equal(got, ref), f"{int((got != ref).sum())} codes differ at gaps >= 1e-6"
        else:
            stats = check_codes(got, x, cb)
            # whatever differs picked the runner-up: nothing but the two planted centroids
            assert stats["n_diff"] <= stats["n"]


def test_10_bit_codes_at_the_boundary():
    fmt = cq.CQFormat(8, 10, 128, 1)
    cb, x = _plant(8, 10, fmt.groups, 128, BAND_EXACT, 77)
    ref = _check_planted(x, cb, BAND_EXACT)
    for B, T in ((1, 128), (8, 16)):
        t_cap = (T + 63) // 64 * 64
        got = cache_to_codes(gpu_encode(x.reshape(B, T, -1), cb, fmt, t_cap), fmt, B, t_cap, T).reshape(B * T, -1)
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("c", [2, 4, 8])
@pytest.mark.parametrize("band", [BAND_EXACT, BAND_LOOSE], ids=["gap_1e-6_to_3e-6", "gap_1e-8_to_1e-6"])
def test_fused_step_encode_at_the_boundary(c, band):
    # the new token of a decode step, key row and value row both planted; 16 sequences, 200 cached tokens
    b, hkv, hq, B, T, t_cap = 8, 1, 2, 16, 200, 256
    fmt = cq.CQFormat(c, b, 128, hkv)
    ck, xk = _plant(c, b, fmt.groups, B, band, 31 * c + 1)
    cv, xv = _plant(c, b, fmt.groups, B, band, 31 * c + 2)
    ref_k, ref_v = _check_planted(xk, ck, band), _check_planted(xv, cv, band)
    rng = np.random.default_rng(9)
    old = rng.integers(0, 256, size=(B, T, fmt.groups)).astype(np.uint16)
    kcache, vcache = codes_to_cache(old, fmt, t_cap), codes_to_cache(old[:, ::-1].copy(), fmt, t_cap)
    q = rng.standard_normal((B, hq, 128)).astype(np.float16)
    cq.cq_decode_step(dev(q), dev(xk), dev(xv), kcache, vcache, dev(ck), dev(cv), 0.1, fmt, T, t_cap)
    torch.cuda.synchronize()
    got_k = cache_to_codes(kcache, fmt, B, t_cap, 1, T - 1).reshape(B, -1)
    got_v = cache_to_codes(vcache, fmt, B, t_cap, 1, T - 1).reshape(B, -1)
    if band is BAND_EXACT:
        assert np.array_equal(got_k, ref_k) and np.array_equal(got_v, ref_v)
    else:
        check_codes(got_k, xk, ck)
        check_codes(got_v, xv, cv)
