"""Pins for the centroid-learning oracle (oracle/kmeans_oracle.c): closed forms, library k-means
implementations started from the same centres, the exact sampling law of k-means++, the weighted
objective of Eq. 6 through point replication, and Eq. 5's objective through the (separately pinned)
encode / dequantize oracle.  None of these re-uses the oracle's own arithmetic."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.cluster.vq
import scipy.stats
from sklearn.cluster import KMeans

from oracle import cq_oracle as O
from oracle import kmeans_oracle as KO


def _blobs(rng, n, c, k, spread=0.05, scale=4.0):
    centres = scale * rng.standard_normal((k, c))
    lab = rng.integers(0, k, size=n)
    return (centres[lab] + spread * rng.standard_normal((n, c))).astype(np.float16), lab, centres


# ------------------------------------------------------------------------------------------
# Lloyd iterations
# ------------------------------------------------------------------------------------------
def test_single_cluster_is_the_exact_mean():
    rng = np.random.default_rng(1)
    x = (3.0 * rng.standard_normal((777, 4))).astype(np.float16)
    cent, assign, _ = KO.lloyd(x, 4, np.zeros((1, 1, 4), np.float32), 1)
    # exact rational mean of the fp16 values, rounded once to binary64 then to binary32
    for ch in range(4):
        tot = sum(Fraction(float(v)) for v in x[:, ch])
        want = np.float32(float(tot / len(x)))
        assert cent[0, 0, ch] == want
    assert not assign.any()


def test_weighted_single_cluster_is_the_exact_weighted_mean():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((300, 2)).astype(np.float16)
    w = rng.integers(1, 50, size=(300, 1)).astype(np.float32)       # integers: represented exactly
    cent, _, _ = KO.lloyd(x, 2, np.zeros((1, 1, 2), np.float32), 1, w)
    for ch in range(2):
        num = sum(Fraction(float(v)) * int(wi) for v, wi in zip(x[:, ch], w[:, 0]))
        want = np.float32(float(num / int(w.sum())))
        assert cent[0, 0, ch] == want


def test_weight_quantisation_keeps_22_bits_of_the_largest_weight():
    # Hand-computed: the largest weight of a group becomes an integer in [2^21, 2^22), so a weight of
    # 2^-21 of the largest is the integer 1 and a weight of 2^-22 of it (or less) is 0 and leaves the mean.
    # Two points, x = 0 with weight 1 and x = 1000 with weight w: the mean is 1000 wq / (2^21 + wq).
    # A scale exponent off by one in either direction moves both answers.
    x = np.array([[0.0], [1000.0]], dtype=np.float16)
    for w_small, wq in ((2.0 ** -21, 1), (2.0 ** -22, 0), (1.5 * 2.0 ** -21, 1), (3.0 * 2.0 ** -21, 3), (2.0 ** -40, 0)):
        w = np.array([[1.0], [w_small]], dtype=np.float32)
        cent, _, _ = KO.lloyd(x, 1, np.zeros((1, 1, 1), np.float32), 1, w)
        want = np.float32(float(Fraction(1000 * wq, 2 ** 21 + wq)))
        assert cent[0, 0, 0] == want, (w_small, cent[0, 0, 0], want)
        assert list(KO.integer_weights(w, 2, 1)[0]) == [2 ** 21, wq]
    # the scale follows the largest weight, whatever its size: 3 * 2^k has the integer 3 * 2^20
    for k in (-30, 0, 17):
        w = np.array([[3.0 * 2.0 ** k], [2.0 ** k]], dtype=np.float32)
        assert list(KO.integer_weights(w, 2, 1)[0]) == [3 * 2 ** 20, 2 ** 20]


def test_weighted_update_against_plain_fp64_eq6_with_weights_over_30_binades():
    # Eq. 6's update in plain fp64 (weighted mean of every cluster with the real-valued weights) against
    # the oracle's integer-weight arithmetic, weights spread over 34 binades (squared gradients span many
    # decades).  Integer weights deviate from w 2^kw by less than one unit, i.e. by less than 2^-21 of
    # the group's largest weight each, so a cluster's mean moves by at most
    # n_cluster 2^-21 w_max spread / W_cluster; clusters that hold a weight within 2^10 of the largest
    # therefore agree to 1e-4 of the spread, which is asserted; the weighted objective (Eq. 6) of the
    # oracle's centroids exceeds that of the plain update by no more than 1e-5 of itself.
    rng = np.random.default_rng(77)
    n, c, k = 4000, 4, 8
    x, lab, _ = _blobs(rng, n, c, k, spread=0.3)
    w = (2.0 ** rng.uniform(-34, 0, size=(n, 1))).astype(np.float32)
    w[:k, 0] = rng.uniform(0.5, 1.0, size=k)                       # every cluster holds a heavy point
    lab[:k] = np.arange(k)
    x[:k] = x[[np.flatnonzero(lab == j)[-1] for j in range(k)]]
    start = np.stack([x[lab == j].astype(np.float64).mean(0) for j in range(k)])[None].astype(np.float32)
    cent, assign, _ = KO.lloyd(x, c, start, 1, w)
    x64, w64 = x.astype(np.float64), w[:, 0].astype(np.float64)
    d = ((x64[:, None, :] - start[0].astype(np.float64)[None]) ** 2).sum(-1)
    a = d.argmin(1)
    assert np.array_equal(a, assign[0])                             # (well separated blobs: no close calls)
    spread = x64.max(0) - x64.min(0)
    obj_plain = obj_oracle = 0.0
    for j in range(k):
        m = a == j
        plain = (w64[m, None] * x64[m]).sum(0) / w64[m].sum()
        assert np.all(np.abs(cent[0, j] - plain) <= 1e-4 * spread + 2.0 ** -22 * np.abs(plain))
        obj_plain += (w64[m] * ((x64[m] - plain) ** 2).sum(-1)).sum()
        obj_oracle += (w64[m] * ((x64[m] - cent[0, j].astype(np.float64)) ** 2).sum(-1)).sum()
    assert obj_plain <= obj_oracle <= obj_plain * (1 + 1e-5)


def test_sampling_scale_keeps_tiny_masses_and_never_overflows():
    # The k-means++ masses are integers floor(p 2^kq) scaled so that their sum over N points stays
    # below 2^62 while the largest keeps about 62 - log2 N bits.  (a) A point whose mass is 2^-40 of the
    # largest still owns an interval: with 4 points the largest mass is 2^59 units and this one 2^19,
    # at the bottom of the range (the point comes first) of 2^60 + 2^19 units in all, so exactly the
    # random words below 2^23 pick it.  A scale one bit off moves that boundary; 20 bits too small
    # would give the point no interval at all.  (b) 2^16 points of equal mass: the random
    # word 2^63 (the middle of the range) picks the middle point; a scale three or more bits too
    # large would overflow the 64-bit sum.
    x = np.zeros((4, 2), dtype=np.float16)
    x[:, 0] = [2.0 ** -10, 0.0, 1024.0, -1024.0]          # first pick: index 1 (the origin), rnd = 2^62
    first = 2 ** 62                                        # floor(2^62 * 4 / 2^64) = 1
    for r1, want in ((2 ** 22, 0), (2 ** 23 - 1, 0), (2 ** 23, 2)):
        picks, _ = KO.kmeanspp(x, 2, 2, np.array([[first, r1]], dtype=np.uint64))
        assert list(picks[0]) == [1, want], (r1, picks)
    n = 2 ** 16
    x = np.zeros((n, 2), dtype=np.float16)
    x[1:, 0] = 1.0                                         # all but the first centre at the same distance
    picks, _ = KO.kmeanspp(x, 2, 2, np.array([[0, 2 ** 63]], dtype=np.uint64))
    assert picks[0, 0] == 0 and picks[0, 1] in (n // 2, n // 2 + 1)


@pytest.mark.parametrize("c", [2, 4, 8])
def test_lloyd_matches_sklearn_and_scipy_from_the_same_centres(c):
    rng = np.random.default_rng(10 + c)
    k, n = 12, 1500
    x, _, _ = _blobs(rng, n, c, k)
    init = x[rng.choice(n, size=k, replace=False)].astype(np.float32)
    cent, assign, obj = KO.lloyd(x, c, init[None], 30)
    xd = x.astype(np.float64)
    sk = KMeans(n_clusters=k, init=init.astype(np.float64), n_init=1, algorithm="lloyd", max_iter=30, tol=0.0).fit(xd)
    # well separated data: no near ties, both reach the same fixed point
    order = np.argsort(sk.cluster_centers_[:, 0])
    mine = np.argsort(cent[0][:, 0])
    assert np.allclose(cent[0][mine], sk.cluster_centers_[order], rtol=0, atol=2e-6 * np.abs(xd).max())
    assert np.array_equal(assign[0], sk.labels_)
    assert obj[0, -1] == pytest.approx(sk.inertia_, rel=1e-5)
    sp_cent, sp_lab = scipy.cluster.vq.kmeans2(xd, init.astype(np.float64), iter=30, minit="matrix")
    assert np.allclose(cent[0], sp_cent, rtol=0, atol=2e-6 * np.abs(xd).max())
    assert np.array_equal(assign[0], sp_lab)


def test_weighted_lloyd_matches_sklearn_sample_weight():
    rng = np.random.default_rng(5)
    k, n, c = 6, 900, 4
    x, _, _ = _blobs(rng, n, c, k, spread=0.4)
    w = rng.integers(1, 9, size=(n, 1)).astype(np.float32)
    init = x[rng.choice(n, size=k, replace=False)].astype(np.float32)
    cent, assign, _ = KO.lloyd(x, c, init[None], 40, w)
    sk = KMeans(n_clusters=k, init=init.astype(np.float64), n_init=1, algorithm="lloyd", max_iter=40, tol=0.0)
    sk.fit(x.astype(np.float64), sample_weight=w[:, 0].astype(np.float64))
    assert np.allclose(cent[0], sk.cluster_centers_, rtol=0, atol=1e-5)
    assert np.array_equal(assign[0], sk.labels_)


def test_integer_weights_equal_point_replication():
    rng = np.random.default_rng(6)
    n, c, k = 400, 2, 5
    x = rng.standard_normal((n, c)).astype(np.float16)
    reps = rng.integers(1, 5, size=n)
    w = reps.astype(np.float32)[:, None]
    init = x[:k].astype(np.float32)[None]
    cw, _, ow = KO.lloyd(x, c, init, 15, w)
    xr = np.repeat(x, reps, axis=0)
    cr, _, orr = KO.lloyd(xr, c, init, 15)
    assert np.array_equal(cw, cr)
    # the weighted run reports the objective in units of its integer weights (largest weight -> [2^21, 2^22))
    wq = KO.integer_weights(w, n, 1)[0]
    unit = wq[0] / reps[0]
    assert np.all(wq == reps * unit)
    assert np.allclose(ow / unit, orr, rtol=1e-12)


def test_equal_weights_change_nothing_and_zero_weights_mean_unweighted():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((256, 8)).astype(np.float16)
    init = x[:7].astype(np.float32).reshape(1, 7, 8)
    base, a0, _ = KO.lloyd(x, 8, init, 8)
    same, a1, _ = KO.lloyd(x, 8, init, 8, np.full((256, 1), 0.37, np.float32))
    zero, a2, _ = KO.lloyd(x, 8, init, 8, np.zeros((256, 1), np.float32))
    assert np.array_equal(base, same) and np.array_equal(base, zero)
    assert np.array_equal(a0, a1) and np.array_equal(a0, a2)


def test_objective_never_increases_and_empty_clusters_keep_their_centroid():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((600, 4)).astype(np.float16)
    init = np.concatenate([x[:9].astype(np.float32), np.full((1, 4), 1000.0, np.float32)])[None]   # one unreachable
    cent, assign, obj = KO.lloyd(x, 4, init, 25)
    assert np.all(np.diff(obj[0]) <= 1e-6 * obj[0, :-1])
    assert np.array_equal(cent[0, 9], init[0, 9]) and not (assign == 9).any()


def test_a_centroid_on_every_distinct_point_gives_zero_objective():
    rng = np.random.default_rng(9)
    pts = rng.standard_normal((16, 2)).astype(np.float16)
    x = pts[rng.integers(0, 16, size=200)]
    cent, assign, obj = KO.lloyd(x, 2, pts.astype(np.float32)[None], 3)
    assert np.all(obj == 0) and np.array_equal(cent[0], pts.astype(np.float32))
    assert np.array_equal(pts[assign[0]], x)


def test_objective_is_eq5_frobenius_error_of_the_encode_oracle():
    rng = np.random.default_rng(11)
    n, D, c, K = 512, 32, 4, 16
    x = rng.standard_normal((n, D)).astype(np.float16)
    rnd = rng.integers(0, 2 ** 64, size=(D // c, K), dtype=np.uint64)
    cent16, _, _, _ = KO.fit(x, c, K, rnd, 10)
    codes = O.encode(x, cent16)
    err = ((x.astype(np.float64) - O.dequantize(codes, cent16)) ** 2).reshape(n, D // c, c).sum((0, 2))
    obj, assign = KO.objective(x, c, cent16.astype(np.float32))
    assert np.allclose(obj, err, rtol=1e-5)
    assert (assign.T != codes).mean() < 0.01            # binary32 vs binary64 near ties only


def test_groups_are_independent_and_follow_the_channel_layout():
    rng = np.random.default_rng(12)
    n, c, K = 300, 4, 8
    xa = rng.standard_normal((n, c)).astype(np.float16)
    xb = (5 + rng.standard_normal((n, c))).astype(np.float16)
    rnd = rng.integers(0, 2 ** 64, size=(2, K), dtype=np.uint64)
    both = KO.fit(np.concatenate([xa, xb], axis=1), c, K, rnd, 6)
    a = KO.fit(xa, c, K, rnd[:1], 6)
    b = KO.fit(xb, c, K, rnd[1:], 6)
    assert np.array_equal(both[1][0], a[1][0]) and np.array_equal(both[1][1], b[1][0])
    assert np.array_equal(both[2][1], b[2][0])


# ------------------------------------------------------------------------------------------
# k-means++
# ------------------------------------------------------------------------------------------
def test_first_pick_is_uniform_in_the_random_word_and_centres_are_the_picked_points():
    rng = np.random.default_rng(20)
    n = 1000
    x = rng.standard_normal((n, 2)).astype(np.float16)
    for r in (0, 1, 2 ** 63, 2 ** 64 - 1, 123456789123456789):
        rnd = np.array([[r, 5, 7]], dtype=np.uint64)
        picks, cent = KO.kmeanspp(x, 2, 3, rnd)
        assert picks[0, 0] == (r * n) >> 64
        assert np.array_equal(cent[0], x[picks[0]].astype(np.float32))


def test_second_pick_follows_the_squared_distance_law():
    # 4 candidate positions at squared distances 0, 1, 4, 9 from where the first centre will be
    pos = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 2.0], [3.0, 0.0]], dtype=np.float16)
    counts = np.array([50, 30, 20, 10])
    x = np.repeat(pos, counts, axis=0)
    rng = np.random.default_rng(21)
    trials = 4000
    hits = np.zeros(4)
    for _ in range(trials):
        r1 = int(rng.integers(0, 2 ** 64, dtype=np.uint64))
        picks, _ = KO.kmeanspp(x, 2, 2, np.array([[0, r1]], dtype=np.uint64))     # first pick: token 0, at the origin
        assert picks[0, 0] == 0
        hits[np.searchsorted(np.cumsum(counts), picks[0, 1], side="right")] += 1
    mass = counts * np.array([0.0, 1.0, 4.0, 9.0])
    assert hits[0] == 0
    chi = scipy.stats.chisquare(hits[1:], trials * mass[1:] / mass.sum())
    assert chi.pvalue > 1e-3


def test_weighted_first_pick_follows_the_weights():
    x = np.zeros((4, 2), dtype=np.float16)
    x[:, 0] = [0, 1, 2, 3]
    w = np.array([[1.0], [0.0], [2.0], [5.0]], dtype=np.float32)
    rng = np.random.default_rng(22)
    hits = np.zeros(4)
    for _ in range(4000):
        r0 = int(rng.integers(0, 2 ** 64, dtype=np.uint64))
        picks, _ = KO.kmeanspp(x, 2, 1, np.array([[r0]], dtype=np.uint64), w)
        hits[picks[0, 0]] += 1
    assert hits[1] == 0
    chi = scipy.stats.chisquare(hits[[0, 2, 3]], 4000 * np.array([1, 2, 5]) / 8)
    assert chi.pvalue > 1e-3


def test_sampling_boundaries_are_exact():
    # two far points of equal mass: the pick flips exactly where rnd crosses the middle of the range
    x = np.array([[0.0, 0.0], [1.0, 0.0], [-1.0, 0.0]], dtype=np.float16)
    for r1, want in ((2 ** 63 - 1, 1), (2 ** 63, 2), (0, 1), (2 ** 64 - 1, 2)):
        picks, _ = KO.kmeanspp(x, 2, 2, np.array([[0, r1]], dtype=np.uint64))
        assert list(picks[0]) == [0, want]


def test_all_points_identical_falls_back_to_uniform_picks():
    x = np.full((50, 4), 1.5, dtype=np.float16)
    rnd = np.array([[2 ** 63, 2 ** 62, 3 * 2 ** 62]], dtype=np.uint64)
    picks, cent = KO.kmeanspp(x, 4, 3, rnd)
    assert list(picks[0]) == [25, 12, 37]
    assert np.all(cent == 1.5)


def test_kmeanspp_then_lloyd_beats_random_codebooks_on_correlated_data():
    import synth
    r = synth.tensor_recipe(3, 0, "k", 128)
    x = synth.sample_activations(r, 2048, 0)
    K, c = 64, 8
    rng = np.random.default_rng(23)
    rnd = rng.integers(0, 2 ** 64, size=(128 // c, K), dtype=np.uint64)
    _, cent, _, obj = KO.fit(x, c, K, rnd, 20)
    sampled = synth.sample_codebook(r, c, 8)[:, :K].astype(np.float32)
    base, _ = KO.objective(x, c, sampled)
    assert np.all(obj[:, -1] < 0.8 * base)


def test_more_coupled_channels_lower_the_error_at_equal_bits_per_channel():
    """The trend of the paper's ablation on coupled channels (Section 4.3, Figure 4) on the
    correlated synthetic activations: at a fixed bit budget per channel the learned codebooks'
    quantization error (Eq. 5) falls as more channels are coupled."""
    import synth
    D, n = 16, 6000
    x = synth.sample_activations(synth.tensor_recipe(7, 0, "v", D), n)
    rng = np.random.default_rng(5)

    def err(c, b):
        K = 1 << b
        rnd = rng.integers(0, 2 ** 64, size=(D // c, K), dtype=np.uint64)
        _, cent, _, obj = KO.fit(x, c, K, rnd, 25)
        total, _ = KO.objective(x, c, cent)
        return float(total.sum())
    one_bit = [err(2, 2), err(4, 4), err(8, 8)]            # 1 bit per channel
    two_bits = [err(1, 2), err(2, 4), err(4, 8)]           # 2 bits per channel
    assert one_bit[0] > one_bit[1] > one_bit[2]
    assert two_bits[0] > two_bits[1] > two_bits[2]
    assert two_bits[2] < one_bit[2]                        # and more bits help at equal coupling
