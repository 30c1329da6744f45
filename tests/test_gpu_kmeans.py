"""GPU parity of the centroid learning (cq_kmeans_fit, through the C ABI) against its CPU oracle:
every pick of k-means++, every fp32 centroid after every tested number of Lloyd iterations and
every assignment must be IDENTICAL (both sides take each decision in the same arithmetic; sums are
exact integers), on sizes that are not multiples of any tile, with and without Eq. 6 weights."""
import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq
import synth
from oracle import cq_oracle as O
from oracle import kmeans_oracle as KO

pytestmark = pytest.mark.gpu


def _data(seed, n, D, which="k"):
    r = synth.tensor_recipe(40 + seed, 0, which, D)
    return synth.sample_activations(r, n, 0)


def _rnd(seed, G, K):
    return np.random.default_rng(seed).integers(0, 2 ** 64, size=(G, K), dtype=np.uint64)


def _dev_rnd(rnd):
    return torch.from_numpy(rnd.view(np.int64)).cuda()


def _weights(seed, n, G, zero_fraction=0.1):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((n, G)) ** 2 * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)   # gradient-square like
    w[rng.random((n, G)) < zero_fraction] = 0.0
    return w


@pytest.mark.parametrize("c,b,n", [(8, 8, 1000), (4, 8, 2500), (2, 8, 700), (8, 10, 3000),
                                   (1, 2, 900), (2, 2, 333), (1, 4, 1100), (2, 4, 2000), (4, 4, 650)])
@pytest.mark.parametrize("weighted", [False, True])
def test_kmeanspp_picks_are_the_oracles(c, b, n, weighted):
    fmt = cq.CQFormat(c, b, 128, 1)
    G, K = fmt.groups, 1 << b
    x = _data(c + b, n, 128)
    rnd = _rnd(c * 100 + n, G, K)
    w = _weights(n, n, G) if weighted else None
    picks, cent = KO.kmeanspp(x, c, K, rnd, w)
    out = cq.cq_kmeans_fit(torch.from_numpy(x).cuda(), fmt, 0, rnd=_dev_rnd(rnd),
                           weights=None if w is None else torch.from_numpy(w).cuda(), want_picks=True)
    torch.cuda.synchronize()
    assert np.array_equal(out["picks"].cpu().numpy(), picks)
    assert np.array_equal(out["centroids_f32"].cpu().numpy(), cent)
    assert np.array_equal(out["centroids"].cpu().numpy(), cent.astype(np.float16))


@pytest.mark.parametrize("c,b,n", [(8, 8, 1500), (4, 8, 3001), (2, 8, 640), (8, 10, 2100),
                                   (1, 2, 777), (2, 2, 1500), (1, 4, 640), (2, 4, 901), (4, 4, 3001)])
@pytest.mark.parametrize("weighted", [False, True])
def test_lloyd_iterations_are_bit_identical(c, b, n, weighted):
    fmt = cq.CQFormat(c, b, 128, 2)
    G, K = fmt.groups, 1 << b
    x = _data(2 * c + b, n, 256, "v")
    rng = np.random.default_rng(n)
    init = np.stack([x.reshape(n, G, c)[rng.choice(n, size=K, replace=n < K), g] for g in range(G)]).astype(np.float32)
    w = _weights(n + 1, n, G) if weighted else None
    xd = torch.from_numpy(x).cuda()
    wd = None if w is None else torch.from_numpy(w).cuda()
    for iters in (1, 4):
        cent, assign, _ = KO.lloyd(x, c, init, iters, w)
        out = cq.cq_kmeans_fit(xd, fmt, iters, init_centroids=torch.from_numpy(init).cuda(), weights=wd, want_assignment=True)
        torch.cuda.synchronize()
        assert np.array_equal(out["assignment"].cpu().numpy().view(np.uint16), assign)
        assert np.array_equal(out["centroids_f32"].cpu().numpy(), cent)


def test_fit_end_to_end_and_learned_codebooks_beat_sampled_ones():
    c, b, n, D = 8, 8, 4096, 256
    fmt = cq.CQFormat(c, b, 128, 2)
    G, K = fmt.groups, 1 << b
    r = synth.tensor_recipe(77, 0, "k", D)
    x = synth.sample_activations(r, n, 0)
    rnd = _rnd(5, G, K)
    want16, want32, assign, obj = KO.fit(x, c, K, rnd, 6)
    out = cq.cq_kmeans_fit(torch.from_numpy(x).cuda(), fmt, 6, rnd=_dev_rnd(rnd), want_assignment=True)
    torch.cuda.synchronize()
    got16 = out["centroids"].cpu().numpy()
    assert np.array_equal(got16, want16)
    assert np.array_equal(out["centroids_f32"].cpu().numpy(), want32)
    assert np.array_equal(out["assignment"].cpu().numpy().view(np.uint16), assign)
    # the learned fp16 codebook plugs into cq_encode; Eq. 5's error with it is far below a sampled codebook's
    def frob(cb):
        codes = O.encode(x, cb)
        return ((x.astype(np.float64) - O.dequantize(codes, cb)) ** 2).sum()
    assert frob(got16) < 0.7 * frob(synth.sample_codebook(r, c, b))


def test_fewer_points_than_centroids_identical_points_and_a_single_point():
    c, b = 4, 8
    fmt = cq.CQFormat(c, b, 128, 1)
    G, K = fmt.groups, 256
    cases = [_data(1, 100, 128), np.full((300, 128), 0.75, dtype=np.float16), _data(2, 1, 128)]
    cases.append(np.repeat(_data(3, 8, 128), 40, axis=0))            # 8 distinct points, many exact ties
    for k, x in enumerate(cases):
        n = x.shape[0]
        rnd = _rnd(30 + k, G, K)
        want16, want32, assign, _ = KO.fit(x, c, K, rnd, 3)
        picks, _ = KO.kmeanspp(x, c, K, rnd)
        out = cq.cq_kmeans_fit(torch.from_numpy(x).cuda(), fmt, 3, rnd=_dev_rnd(rnd), want_picks=True, want_assignment=True)
        torch.cuda.synchronize()
        assert np.array_equal(out["picks"].cpu().numpy(), picks), k
        assert np.array_equal(out["centroids_f32"].cpu().numpy(), want32), k
        assert np.array_equal(out["assignment"].cpu().numpy().view(np.uint16), assign), k


def test_strided_rows_and_repeatability():
    c, b, n = 8, 8, 900
    fmt = cq.CQFormat(c, b, 128, 1)
    G, K = fmt.groups, 256
    x = _data(9, n, 128)
    wide = torch.zeros((n, 128 + 64), dtype=torch.float16, device="cuda")
    wide[:, :128] = torch.from_numpy(x).cuda()
    rnd = _dev_rnd(_rnd(9, G, K))
    a = cq.cq_kmeans_fit(wide[:, :128], fmt, 2, rnd=rnd)["centroids_f32"]
    b_ = cq.cq_kmeans_fit(torch.from_numpy(x).cuda(), fmt, 2, rnd=rnd)["centroids_f32"]
    c_ = cq.cq_kmeans_fit(torch.from_numpy(x).cuda(), fmt, 2, rnd=rnd)["centroids_f32"]
    torch.cuda.synchronize()
    assert torch.equal(a, b_) and torch.equal(b_, c_)
