"""Pins for the scoring oracle (Sec. 3.1, Eq. 4-5): closed forms for zero
queries, mass conservation, the link to the attention oracle through one-hot
values, permutation equivariance, beta accumulation, planted keys on top."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
from paper_2508_16201_amd import synth
from paper_2508_16201_amd.synth import f32_to_bf16_bits as to_bf16, bf16_bits_to_f32 as to_f32


def rnd(shape, seed):
    return to_bf16(np.random.default_rng(seed).standard_normal(shape).astype(np.float32))


def test_zero_queries_closed_forms():
    V, L, P, hq, hkv, d = 40, 6, 3, 4, 2, 8
    n_keys = P + V + L
    q = to_bf16(np.zeros((L, hq, d), np.float32))
    k = rnd((n_keys, hkv, d), 0)
    a1 = oracle.score(q, k, P, V, P + V, 0.3, norm_mode=1)
    np.testing.assert_allclose(a1, np.full(V, 1.0 / V), rtol=1e-14)
    a0 = oracle.score(q, k, P, V, P + V, 0.3, norm_mode=0)
    # query i sits at position P+V+i and sees P+V+i+1 keys, all with equal weight
    expect = np.mean([1.0 / (P + V + i + 1) for i in range(L)])
    np.testing.assert_allclose(a0, np.full(V, expect), rtol=1e-14)


def test_mass_conservation_and_complement():
    V, L, P, hq, hkv, d = 50, 7, 2, 4, 2, 16
    n_keys = P + V + L
    q, k = rnd((L, hq, d), 1), rnd((n_keys, hkv, d), 2)
    scale = 0.25
    a1 = oracle.score(q, k, P, V, P + V, scale, norm_mode=1)
    np.testing.assert_allclose(a1.sum(), 1.0, rtol=1e-13)
    a0 = oracle.score(q, k, P, V, P + V, scale, norm_mode=0)
    # mass the same rows put on the non-video columns, from a library softmax
    qf, kf = to_f32(q).astype(np.float64), to_f32(k).astype(np.float64)
    other = 0.0
    for h in range(hq):
        for i in range(L):
            vis = P + V + i + 1
            p = softmax(scale * kf[:vis, h // 2] @ qf[i, h])
            other += p[:P].sum() + p[P + V:].sum()
    other /= hq * L
    assert 0.0 < a0.sum() < 1.0
    np.testing.assert_allclose(a0.sum(), 1.0 - other, rtol=1e-12)
    assert np.all(a0 >= 0) and np.all(a1 >= 0)


def test_matches_attention_oracle_with_one_hot_values_and_lse():
    # tiny: all keys fit in d, so attention over identity values returns M's rows
    d, V, L, P, hq, hkv = 32, 20, 5, 2, 4, 2
    n_keys = P + V + L
    q, k = rnd((L, hq, d), 3), rnd((n_keys, hkv, d), 4)
    v = np.zeros((n_keys, hkv, d), np.float32)
    for j in range(n_keys):
        v[j, :, j] = 1.0
    scale = 1 / np.sqrt(d)
    probs, lse_attn = oracle.decode_attn(q, k, to_bf16(v), scale)   # block = the text rows
    expect = probs[:, :, P:P + V].mean(axis=(0, 1))
    a0, lse = oracle.score(q, k, P, V, P + V, scale, norm_mode=0, want_lse=True)
    np.testing.assert_allclose(a0, expect, rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(lse, lse_attn, rtol=1e-13)
    # video-only normalisation = rows renormalised over the video slice
    sl = probs[:, :, P:P + V]
    expect1 = (sl / sl.sum(axis=-1, keepdims=True)).mean(axis=(0, 1))
    a1 = oracle.score(q, k, P, V, P + V, scale, norm_mode=1)
    np.testing.assert_allclose(a1, expect1, rtol=1e-12, atol=1e-16)


def test_causal_text_prefix_sees_fewer_keys():
    # a text query placed before the last video keys must not score them
    V, L, hq, hkv, d = 12, 3, 2, 1, 8
    q, k = rnd((L, hq, d), 5), rnd((V + L, hkv, d), 6)
    a = oracle.score(q, k, 0, V, V - 4, 0.3, norm_mode=0)      # queries at positions 8, 9, 10
    assert a[11] == 0.0 and a[10] > 0.0 and a[8] > 0.0
    qf, kf = to_f32(q).astype(np.float64), to_f32(k).astype(np.float64)
    col9 = 0.0
    for h in range(hq):
        for i, pos in enumerate((8, 9, 10)):
            p = softmax(0.3 * kf[:pos + 1, 0] @ qf[i, h])
            col9 += p[9] if pos >= 9 else 0.0
    np.testing.assert_allclose(a[9], col9 / (hq * L), rtol=1e-12)


def test_permuting_video_keys_permutes_scores():
    V, L, hq, hkv, d = 30, 4, 4, 2, 16
    q, k = rnd((L, hq, d), 7), rnd((V + L, hkv, d), 8)
    perm = np.random.default_rng(9).permutation(V)
    k2 = k.copy(); k2[:V] = k[:V][perm]
    for mode in (0, 1):
        a = oracle.score(q, k, 0, V, V, 0.25, norm_mode=mode)
        b = oracle.score(q, k2, 0, V, V, 0.25, norm_mode=mode)
        np.testing.assert_allclose(b, a[perm], rtol=1e-12)


def test_beta_accumulates_layers():
    V, L, hq, hkv, d = 16, 3, 2, 1, 8
    q, k = rnd((L, hq, d), 10), rnd((V + L, hkv, d), 11)
    a = oracle.score(q, k, 0, V, V, 0.3)
    b = oracle.score(q, k, 0, V, V, 0.3, beta=1.0, scores_in=a)
    np.testing.assert_allclose(b, 2 * a, rtol=1e-14)
    c = oracle.score(q, k, 0, V, V, 0.3, beta=0.5, scores_in=np.ones(V))
    np.testing.assert_allclose(c, 0.5 + a, rtol=1e-14)


def test_head_mean_not_head_sum_and_group_mapping():
    # q heads 0,1 read kv head 0; heads 2,3 read kv head 1.  Zero the queries of
    # group 1: its rows turn uniform (1/V each in mode 1), group 0's stay peaked.
    V, L, hq, hkv, d = 10, 2, 4, 2, 8
    q = to_f32(rnd((L, hq, d), 12)); q[:, 2:, :] = 0
    k = rnd((V + L, hkv, d), 13)
    a = oracle.score(to_bf16(q), k, 0, V, V, 0.5, norm_mode=1)
    qf, kf = q.astype(np.float64), to_f32(k).astype(np.float64)
    g0 = np.mean([softmax(0.5 * kf[:V, 0] @ qf[i, h]) for i in range(L) for h in (0, 1)], axis=0)
    np.testing.assert_allclose(a, 0.5 * g0 + 0.5 / V, rtol=1e-12)


@pytest.mark.parametrize("w", [synth.TINY])
def test_planted_keys_rank_first_and_long_tail(w):
    """Generator self-test through the oracle: every planted key outranks every
    other token, and the top 10 % of tokens hold more than half of the score
    mass (the long tail of Sec. 3.2)."""
    t = synth.make_layer(w)
    a = oracle.score(t["q_text"], t["k"][:w.n_ctx], 0, w.n_video, w.n_video, w.softmax_scale)
    planted = np.zeros(w.n_video, bool); planted[t["planted"]] = True
    assert a[planted].min() > a[~planted].max()
    top = np.sort(a)[::-1][: w.n_video // 10]
    assert top.sum() > 0.5 * a.sum()


def test_rejects_bad_arguments():
    q, k = rnd((2, 2, 8), 14), rnd((6, 1, 8), 15)
    with pytest.raises(ValueError):
        oracle.score(q, k, 3, 4, 6, 0.3)          # video span beyond the keys
    with pytest.raises(ValueError):
        oracle.score(q, k, 0, 4, 4, 0.3, norm_mode=2)
