"""The seeded input generator: determinism and the statistics its recipe promises.  CPU only."""
import numpy as np

import synth


def test_mixing_block_gives_unit_variance_and_0p7_correlation():
    L = synth.mixing_block()
    cov = L @ L.T
    assert np.allclose(np.diag(cov), 1.0)
    off = cov[~np.eye(8, dtype=bool)]
    assert np.allclose(off, 0.7)


def test_streams_are_deterministic_and_distinct():
    r = synth.tensor_recipe(1, 0, "k", 256)
    a = synth.sample_activations(r, 32)
    assert np.array_equal(a, synth.sample_activations(r, 32))
    assert not np.array_equal(a, synth.sample_activations(r, 32, chunk=1))
    rv = synth.tensor_recipe(1, 0, "v", 256)
    assert not np.array_equal(a, synth.sample_activations(rv, 32))
    assert a.dtype == np.float16 and a.shape == (32, 256)


def test_key_outlier_channels_and_sample_statistics():
    D = 1024
    rk = synth.tensor_recipe(3, 0, "k", D)
    rv = synth.tensor_recipe(3, 0, "v", D)
    assert int((rk.channel_scale == 10).sum()) == round(0.04 * D) == 41
    assert np.all(rv.channel_scale == 1)
    x = synth.sample_activations(rv, 20000).astype(np.float64) - rv.bias
    corr = np.corrcoef(x[:, :16].T)
    assert np.allclose(corr[:8, :8][~np.eye(8, dtype=bool)], 0.7, atol=0.03)
    assert np.allclose(corr[:8, 8:], 0.0, atol=0.04)
    assert np.allclose(x.std(0), 1.0, atol=0.05)


def test_configs_follow_the_named_workloads():
    c = synth.CONFIGS
    assert (c[1].c, c[1].b, c[1].n_groups, c[1].context) == (8, 8, 512, 1024)
    assert (c[2].c, c[2].n_groups, c[2].batch, c[2].layers) == (4, 1024, 16, 32)
    assert (c[3].c, c[3].n_groups, c[3].batch, c[3].context) == (2, 2048, 64, 8192)
    assert (c[4].b, c[4].n_kv_heads, c[4].n_groups, c[4].n_centroids) == (10, 8, 128, 1024)
    assert (c[5].context, c[5].encode_tokens) == (131072, 32768)
