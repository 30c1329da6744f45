"""Pins for the oracle's decode attention (Eq. 1 of the paper over dequantized K/V):
library attention, pure-Python brute force, closed forms and invariants.  CPU only."""
import math

import numpy as np
import pytest

from oracle import cq_oracle as O


def _case(seed, B, Hq, Hkv, d, T, c, b):
    rng = np.random.default_rng(seed)
    G = Hkv * d // c
    K = 1 << b
    q = rng.standard_normal((B, Hq, d)).astype(np.float16)
    ck = rng.standard_normal((G, K, c)).astype(np.float16)
    cv = rng.standard_normal((G, K, c)).astype(np.float16)
    kc = rng.integers(0, K, size=(B, T, G)).astype(np.uint16)
    vc = rng.integers(0, K, size=(B, T, G)).astype(np.uint16)
    return q, kc, vc, ck, cv


def _dequant_np(codes, cb):
    """[B, T, G] codes -> [B, T, G*c] by numpy indexing (independent of the C code)."""
    B, T, G = codes.shape
    c = cb.shape[2]
    out = np.empty((B, T, G, c))
    for g in range(G):
        out[:, :, g, :] = cb[g].astype(np.float64)[codes[:, :, g]]
    return out.reshape(B, T, G * c)


def test_attention_equals_pure_python_dequantize_then_attend():
    B, Hq, Hkv, d, T, c, b = 2, 2, 2, 4, 5, 2, 3
    q, kc, vc, ck, cv = _case(1, B, Hq, Hkv, d, T, c, b)
    scale = 0.37
    out = O.attention(q, kc, vc, ck, cv, scale, Hkv)
    Gh = d // c
    for n in range(B):
        for h in range(Hq):
            ks, vs = [], []
            for t in range(T):
                krow, vrow = [], []
                for gl in range(Gh):
                    g = h * Gh + gl
                    krow += [float(v) for v in ck[g, kc[n, t, g]]]
                    vrow += [float(v) for v in cv[g, vc[n, t, g]]]
                ks.append(krow)
                vs.append(vrow)
            s = [scale * sum(float(q[n, h, i]) * ks[t][i] for i in range(d)) for t in range(T)]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            z = sum(e)
            for i in range(d):
                want = sum(e[t] / z * vs[t][i] for t in range(T))
                assert out[n, h, i] == pytest.approx(want, rel=1e-13, abs=1e-15)


@pytest.mark.parametrize("Hq,Hkv,c,b", [(4, 4, 8, 8), (8, 2, 4, 8), (4, 1, 8, 10), (2, 2, 2, 8)])
def test_attention_equals_torch_sdpa_on_dequantized_kv(Hq, Hkv, c, b):
    import torch
    import torch.nn.functional as F
    B, d, T = 2, 16, 37
    q, kc, vc, ck, cv = _case(5, B, Hq, Hkv, d, T, c, b)
    scale = 1.0 / math.sqrt(d)
    out = O.attention(q, kc, vc, ck, cv, scale, Hkv)
    kh = _dequant_np(kc, ck).reshape(B, T, Hkv, d).transpose(0, 2, 1, 3)      # [B, Hkv, T, d]
    vh = _dequant_np(vc, cv).reshape(B, T, Hkv, d).transpose(0, 2, 1, 3)
    rep = Hq // Hkv
    kh = np.repeat(kh, rep, axis=1)     # query head h uses KV head h // rep
    vh = np.repeat(vh, rep, axis=1)
    qq = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    want = F.scaled_dot_product_attention(qq, torch.from_numpy(kh), torch.from_numpy(vh), scale=scale)
    np.testing.assert_allclose(out, want[:, :, 0, :].numpy(), rtol=1e-11, atol=1e-13)


def test_single_token_context_returns_its_dequantized_value_exactly():
    B, Hq, Hkv, d, T, c, b = 3, 4, 2, 8, 1, 4, 8
    q, kc, vc, ck, cv = _case(2, B, Hq, Hkv, d, T, c, b)
    out = O.attention(q, kc, vc, ck, cv, 0.5, Hkv)
    v0 = _dequant_np(vc, cv).reshape(B, Hkv, d)
    for h in range(Hq):
        assert np.array_equal(out[:, h], v0[:, h // (Hq // Hkv)])


def test_all_tokens_sharing_one_value_code_return_that_centroid():
    B, Hq, Hkv, d, T, c, b = 1, 2, 2, 8, 50, 8, 8
    q, kc, vc, ck, cv = _case(3, B, Hq, Hkv, d, T, c, b)
    vc[:] = vc[:, :1]
    out = O.attention(q, kc, vc, ck, cv, 0.2, Hkv)
    want = _dequant_np(vc[:, :1], cv).reshape(B, Hkv, d)
    np.testing.assert_allclose(out, want, rtol=1e-14, atol=1e-15)


def test_zero_query_gives_uniform_weights_and_the_code_histogram_average():
    B, Hq, Hkv, d, T, c, b = 1, 2, 2, 8, 200, 4, 4
    q, kc, vc, ck, cv = _case(4, B, Hq, Hkv, d, T, c, b)
    q[:] = 0
    out, probs = O.attention(q, kc, vc, ck, cv, 1.0, Hkv, want_probs=True)
    assert np.allclose(probs, 1.0 / T, rtol=1e-15)
    Gh, K = d // c, 1 << b
    for h in range(Hq):
        for gl in range(Gh):
            g = h * Gh + gl
            counts = np.bincount(vc[0, :, g], minlength=K).astype(np.float64)
            want = (counts[:, None] / T * cv[g].astype(np.float64)).sum(0)
            np.testing.assert_allclose(out[0, h, gl * c:(gl + 1) * c], want, rtol=1e-12, atol=1e-14)


def test_weights_sum_to_one_and_scores_are_lookup_table_sums():
    B, Hq, Hkv, d, T, c, b = 2, 4, 2, 16, 33, 4, 8
    q, kc, vc, ck, cv = _case(6, B, Hq, Hkv, d, T, c, b)
    scale = 0.25
    out, scores, probs = O.attention(q, kc, vc, ck, cv, scale, Hkv, want_scores=True, want_probs=True)
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=1e-14)
    assert np.all(probs >= 0)
    # q . dequant(k) == sum over groups of (q_g . centroid) looked up by code
    Gh = d // c
    rep = Hq // Hkv
    qf = q.astype(np.float64)
    for n in range(B):
        for h in range(Hq):
            hk = h // rep
            lut = np.einsum("gi,gji->gj", qf[n, h].reshape(Gh, c),
                            ck[hk * Gh:(hk + 1) * Gh].astype(np.float64))       # [Gh, K]
            codes = kc[n, :, hk * Gh:(hk + 1) * Gh]                             # [T, Gh]
            want = scale * lut[np.arange(Gh)[None, :], codes].sum(-1)
            np.testing.assert_allclose(scores[n, h], want, rtol=1e-12, atol=1e-13)
    # and the output is the probability-weighted sum of dequantized values
    vh = _dequant_np(vc, cv).reshape(B, T, Hkv, d)
    for h in range(Hq):
        want = np.einsum("bt,btd->bd", probs[:, h], vh[:, :, h // rep])
        np.testing.assert_allclose(out[:, h], want, rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    B, Hq, Hkv, d, T, c, b = 2, 8, 2, 8, 20, 4, 8
    q, kc, vc, ck, cv = _case(7, B, Hq, Hkv, d, T, c, b)
    out = O.attention(q, kc, vc, ck, cv, 0.3, Hkv)
    rep, Gh = Hq // Hkv, d // c
    dup = lambda a, axis: np.repeat(a.reshape(*a.shape[:axis], Hkv, Gh, *a.shape[axis + 1:]), rep, axis=axis) \
        .reshape(*a.shape[:axis], Hq * Gh, *a.shape[axis + 1:])
    out2 = O.attention(q, dup(kc, 2), dup(vc, 2), dup(ck, 0), dup(cv, 0), 0.3, Hq)
    assert np.array_equal(out, out2)


def test_token_permutation_and_ragged_lengths():
    B, Hq, Hkv, d, T, c, b = 2, 2, 2, 8, 40, 4, 8
    q, kc, vc, ck, cv = _case(8, B, Hq, Hkv, d, T, c, b)
    out = O.attention(q, kc, vc, ck, cv, 0.3, Hkv)
    perm = np.random.default_rng(0).permutation(T)
    out_p = O.attention(q, kc[:, perm], vc[:, perm], ck, cv, 0.3, Hkv)
    np.testing.assert_allclose(out_p, out, rtol=1e-12, atol=1e-14)
    lens = np.array([13, 40], dtype=np.int32)
    out_r = O.attention(q, kc, vc, ck, cv, 0.3, Hkv, seq_lens=lens)
    for n in range(B):
        want = O.attention(q[n:n + 1], kc[n:n + 1, :lens[n]], vc[n:n + 1, :lens[n]], ck, cv, 0.3, Hkv)
        assert np.array_equal(out_r[n], want[0])
    with pytest.raises(ValueError):
        O.attention(q, kc, vc, ck, cv, 0.3, Hkv, seq_lens=np.array([0, 40], dtype=np.int32))


def test_large_scores_do_not_overflow():
    B, Hq, Hkv, d, T, c, b = 1, 1, 1, 8, 16, 8, 4
    q, kc, vc, ck, cv = _case(9, B, Hq, Hkv, d, T, c, b)
    kc[0, :, 0] = np.random.default_rng(1).permutation(T)   # distinct keys: a unique arg-max
    out = O.attention(q, kc, vc, ck, cv, 4000.0, Hkv)       # scores of order 1e4
    assert np.all(np.isfinite(out))
    # softmax saturates on the arg-max token
    _, scores = O.attention(q, kc, vc, ck, cv, 4000.0, Hkv, want_scores=True)
    t_star = int(np.argmax(scores[0, 0]))
    want = _dequant_np(vc, cv)[0, t_star]
    np.testing.assert_allclose(out[0, 0], want, rtol=1e-9, atol=1e-12)


# ------------------------------------------------------------------------------------------
# keys cached before the rotary position embedding
# ------------------------------------------------------------------------------------------
def _rope_case(seed, T=37, hq=2, hkv=1, c=8, b=4):
    rng = np.random.default_rng(seed)
    d, K = 128, 1 << b
    G = hkv * d // c
    ck = rng.standard_normal((G, K, c)).astype(np.float16)
    cv = rng.standard_normal((G, K, c)).astype(np.float16)
    kc = rng.integers(0, K, size=(1, T, G)).astype(np.uint16)
    vc = rng.integers(0, K, size=(1, T, G)).astype(np.uint16)
    q = rng.standard_normal((1, hq, d)).astype(np.float16)
    return q, kc, vc, ck, cv


def _rotate_complex(x, pos, base):
    """Rotary embedding through complex numbers: (x_i + j x_{i+d/2}) * exp(j pos theta_i)."""
    d = x.shape[-1]
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    z = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * np.asarray(pos)[..., None] * theta)
    return np.concatenate([z.real, z.imag], axis=-1)


def test_rope_scores_match_the_complex_number_form():
    q, kc, vc, ck, cv = _rope_case(1)
    _, scores = O.attention(q, kc, vc, ck, cv, 0.3, 1, want_scores=True, rope_base=10000.0, pos_offset=5)
    khat = O.dequantize(kc[0], ck)                                  # [T, 128], pre-rotation
    krot = _rotate_complex(khat, np.arange(kc.shape[1]) + 5, 10000.0)
    want = 0.3 * np.einsum("hd,td->ht", q[0].astype(np.float64), krot)
    assert np.allclose(scores[0], want, rtol=1e-12, atol=1e-12)


def test_rope_output_is_plain_attention_over_rotated_keys():
    # rotating the dequantized keys by hand and running textbook softmax attention
    q, kc, vc, ck, cv = _rope_case(2, T=50, hq=4, hkv=2)
    out = O.attention(q, kc, vc, ck, cv, 0.2, 2, rope_base=500.0)
    khat = O.dequantize(kc[0], ck).reshape(50, 2, 128)
    vhat = O.dequantize(vc[0], cv).reshape(50, 2, 128)
    for h in range(4):
        kr = _rotate_complex(khat[:, h // 2], np.arange(50), 500.0)
        s = 0.2 * kr @ q[0, h].astype(np.float64)
        p = np.exp(s - s.max())
        p /= p.sum()
        assert np.allclose(out[0, h], p @ vhat[:, h // 2], rtol=1e-11, atol=1e-12)


def test_rope_depends_on_relative_positions_only():
    # q0 rotated to position p against keys at t + off  ==  q0 rotated to p + s against keys at t + off + s
    q, kc, vc, ck, cv = _rope_case(3)
    q0 = q.astype(np.float64)
    outs = []
    for shift in (0, 11, 1000):
        qrot = _rotate_complex(q0, np.full(q0.shape[:2], 40 + shift), 10000.0)
        q16 = qrot.astype(np.float16)
        # the comparison needs the same fp16 query: rotate in fp64 and feed the fp64 scores directly
        _, s = O.attention(q16, kc, vc, ck, cv, 1.0, 1, want_scores=True, rope_base=10000.0, pos_offset=shift)
        khat = O.dequantize(kc[0], ck)
        krot = _rotate_complex(khat, np.arange(kc.shape[1]) + shift, 10000.0)
        outs.append(np.einsum("hd,td->ht", qrot[0], krot))
        assert np.allclose(s[0], np.einsum("hd,td->ht", q16[0].astype(np.float64), krot), rtol=1e-12, atol=1e-12)
    assert np.allclose(outs[0], outs[1], rtol=1e-9, atol=1e-9) and np.allclose(outs[0], outs[2], rtol=1e-9, atol=1e-9)


def test_rope_at_position_zero_and_norms():
    q, kc, vc, ck, cv = _rope_case(4, T=1)
    plain = O.attention(q, kc, vc, ck, cv, 0.5, 1, want_scores=True)
    roped = O.attention(q, kc, vc, ck, cv, 0.5, 1, want_scores=True, rope_base=10000.0, pos_offset=0)
    assert np.array_equal(plain[1], roped[1]) and np.array_equal(plain[0], roped[0])     # angle 0: identity
    # a rotation preserves the norm of every pair: with q = the rotated key itself the score is |k|^2
    q2, kc2, vc2, ck2, cv2 = _rope_case(5, T=9, hq=1)
    khat = O.dequantize(kc2[0], ck2)
    for t in (0, 3, 8):
        qk = _rotate_complex(khat[t], t + 7, 10000.0)
        # exact fp64 route: compare through the complex form (fp16 rounding of q would blur it)
        assert np.isclose((qk ** 2).sum(), (khat[t] ** 2).sum(), rtol=1e-12)


def test_rope_matches_the_rotate_half_formulation_in_torch():
    import torch
    q, kc, vc, ck, cv = _rope_case(6, T=20)
    _, scores = O.attention(q, kc, vc, ck, cv, 1.0, 1, want_scores=True, rope_base=10000.0)
    k = torch.from_numpy(O.dequantize(kc[0], ck))
    d = 128
    inv_freq = 1.0 / (10000.0 ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    freqs = torch.outer(torch.arange(20, dtype=torch.float64), inv_freq)
    emb = torch.cat([freqs, freqs], dim=-1)
    rot_half = torch.cat([-k[:, d // 2:], k[:, :d // 2]], dim=-1)
    k_rot = k * emb.cos() + rot_half * emb.sin()
    want = torch.from_numpy(q[0].astype(np.float64)) @ k_rot.T
    assert np.allclose(scores[0], want.numpy(), rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------------------
# causal attention of the last m tokens over the coded cache (chunk_attention)
# ------------------------------------------------------------------------------------------
def _chunk_case(seed, B, m, Hq, Hkv, d, T, c, b):
    q1, kc, vc, ck, cv = _case(seed, B, Hq, Hkv, d, T, c, b)
    q = np.random.default_rng(seed + 50).standard_normal((B, m, Hq, d)).astype(np.float16)
    return q, kc, vc, ck, cv


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2)])
def test_chunk_attention_equals_torch_sdpa_with_a_causal_mask(Hq, Hkv):
    import torch
    B, m, d, T, c, b = 2, 7, 16, 23, 4, 4
    q, kc, vc, ck, cv = _chunk_case(31, B, m, Hq, Hkv, d, T, c, b)
    scale = 0.21
    out = O.chunk_attention(q, kc, vc, ck, cv, scale, Hkv)
    k = torch.from_numpy(_dequant_np(kc, ck)).reshape(B, T, Hkv, d).permute(0, 2, 1, 3)
    v = torch.from_numpy(_dequant_np(vc, cv)).reshape(B, T, Hkv, d).permute(0, 2, 1, 3)
    rep = Hq // Hkv
    k, v = k.repeat_interleave(rep, dim=1), v.repeat_interleave(rep, dim=1)
    qt = torch.from_numpy(q.astype(np.float64)).permute(0, 2, 1, 3)               # [B, Hq, m, d]
    # query j sits at position T - m + j: it sees tokens 0 .. T - m + j
    mask = torch.arange(T)[None, :] <= (T - m + torch.arange(m))[:, None]
    want = torch.nn.functional.scaled_dot_product_attention(qt, k, v, attn_mask=mask, scale=scale)
    assert np.allclose(out, want.permute(0, 2, 1, 3).numpy(), rtol=1e-12, atol=1e-13)


def test_chunk_attention_over_pre_rotation_keys_equals_torch_sdpa_over_rotated_keys():
    # the keys rotated by hand (complex-number form) and a library attention with the causal mask
    import torch
    B, m, Hq, Hkv, d, T, c, b = 2, 5, 4, 2, 128, 19, 8, 4
    q, kc, vc, ck, cv = _chunk_case(33, B, m, Hq, Hkv, d, T, c, b)
    scale, base = 0.11, 10000.0
    out = O.chunk_attention(q, kc, vc, ck, cv, scale, Hkv, rope_base=base)
    khat = _dequant_np(kc, ck).reshape(B, T, Hkv, d)
    krot = _rotate_complex(khat, np.arange(T)[None, :, None], base)
    k = torch.from_numpy(krot).permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    v = torch.from_numpy(_dequant_np(vc, cv)).reshape(B, T, Hkv, d).permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    qt = torch.from_numpy(q.astype(np.float64)).permute(0, 2, 1, 3)
    mask = torch.arange(T)[None, :] <= (T - m + torch.arange(m))[:, None]
    want = torch.nn.functional.scaled_dot_product_attention(qt, k, v, attn_mask=mask, scale=scale)
    assert np.allclose(out, want.permute(0, 2, 1, 3).numpy(), rtol=1e-11, atol=1e-12)
    # and it is not the position-independent result
    assert not np.allclose(out, O.chunk_attention(q, kc, vc, ck, cv, scale, Hkv), rtol=1e-3, atol=1e-3)


def test_chunk_attention_special_cases():
    B, m, Hq, Hkv, d, T, c, b = 2, 5, 2, 2, 8, 11, 2, 3
    q, kc, vc, ck, cv = _chunk_case(32, B, m, Hq, Hkv, d, T, c, b)
    out = O.chunk_attention(q, kc, vc, ck, cv, 0.3, Hkv)
    # the last query is plain decode attention over the whole cache, the first sees T - m + 1 tokens
    assert np.array_equal(out[:, -1], O.attention(np.ascontiguousarray(q[:, -1]), kc, vc, ck, cv, 0.3, Hkv))
    first = O.attention(np.ascontiguousarray(q[:, 0]), kc[:, :T - m + 1], vc[:, :T - m + 1], ck, cv, 0.3, Hkv)
    assert np.allclose(out[:, 0], first, rtol=1e-13, atol=0)
    # m = T: the first query sees only token 0 and returns its dequantized value exactly
    qT = np.random.default_rng(5).standard_normal((B, T, Hq, d)).astype(np.float16)
    full = O.chunk_attention(qT, kc, vc, ck, cv, 0.3, Hkv)
    v0 = _dequant_np(vc[:, :1], cv).reshape(B, Hkv, d)
    assert np.array_equal(full[:, 0], v0)
    # ragged: each sequence's chunk ends at its own length; tokens behind it are never read
    lens = np.array([11, 6], dtype=np.int32)
    rag = O.chunk_attention(q, kc, vc, ck, cv, 0.3, Hkv, seq_lens=lens)
    assert np.array_equal(rag[0], out[0])
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[1, 6:], vc2[1, 6:] = 0, 0
    assert np.array_equal(O.chunk_attention(q, kc2, vc2, ck, cv, 0.3, Hkv, seq_lens=lens)[1], rag[1])
    short = O.chunk_attention(q[1:], kc[1:, :6], vc[1:, :6], ck, cv, 0.3, Hkv)
    assert np.allclose(rag[1], short[0], rtol=1e-13, atol=0)
    with pytest.raises(ValueError):
        O.chunk_attention(q, kc, vc, ck, cv, 0.3, Hkv, seq_lens=np.array([11, 4], dtype=np.int32))   # shorter than the chunk
