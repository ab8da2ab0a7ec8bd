"""Pins for the attention oracle (Sec. 2.1: draft decode and parallel
verification): closed forms, special cases that reduce to a library softmax,
and invariants.  None of them re-types the oracle's loop."""
import numpy as np
import pytest
from scipy.special import softmax, expit

import oracle
from paper_2508_16201_amd.synth import f32_to_bf16_bits as to_bf16, bf16_bits_to_f32 as to_f32


def rnd(shape, seed):
    return to_bf16(np.random.default_rng(seed).standard_normal(shape).astype(np.float32))


def test_single_visible_key_returns_its_value():
    q, k, v = rnd((1, 4, 8), 0), rnd((1, 2, 8), 1), rnd((1, 2, 8), 2)
    out, lse = oracle.decode_attn(q, k, v, 0.3)
    vf = to_f32(v).astype(np.float64)
    for h in range(4):
        np.testing.assert_allclose(out[0, h], vf[0, h // 2], rtol=0, atol=0)
    # lse of one key is its logit
    qf, kf = to_f32(q).astype(np.float64), to_f32(k).astype(np.float64)
    np.testing.assert_allclose(lse[0, 3], 0.3 * qf[0, 3] @ kf[0, 1], rtol=1e-14)


def test_identical_keys_give_mean_value():
    k1 = rnd((1, 1, 16), 3)
    k = np.repeat(k1, 37, axis=0)
    v = rnd((37, 1, 16), 4)
    q = rnd((1, 3, 16), 5)
    out, _ = oracle.decode_attn(q, k, v, 0.25)
    mean = to_f32(v).astype(np.float64).mean(axis=0)[0]
    for h in range(3):
        np.testing.assert_allclose(out[0, h], mean, rtol=1e-13, atol=1e-15)


def test_two_keys_sigmoid_closed_form():
    d = 8
    q = np.zeros((1, 1, d), np.float32); q[0, 0, 0] = 2.0
    k = np.zeros((2, 1, d), np.float32); k[0, 0, 0] = 1.5     # logits: scale*3, 0
    v = np.zeros((2, 1, d), np.float32); v[0, 0, :] = 1.0; v[1, 0, :] = -1.0
    scale = 0.5
    out, lse = oracle.decode_attn(to_bf16(q), to_bf16(k), to_bf16(v), scale)
    p0 = expit(scale * 3.0)
    np.testing.assert_allclose(out[0, 0], np.full(d, p0 - (1 - p0)), rtol=1e-14)
    np.testing.assert_allclose(lse[0, 0], np.logaddexp(scale * 3.0, 0.0), rtol=1e-14)


def test_one_hot_values_expose_probabilities_vs_library_softmax():
    # kv_len <= d so V can be the identity: the output row IS the probability row.
    d, kv_len, q_len, hq, hkv = 32, 24, 4, 6, 2
    q, k = rnd((q_len, hq, d), 6), rnd((kv_len, hkv, d), 7)
    v = np.zeros((kv_len, hkv, d), np.float32)
    for j in range(kv_len):
        v[j, :, j] = 1.0
    scale = 1 / np.sqrt(d)
    out, lse = oracle.decode_attn(q, k, to_bf16(v), scale)
    qf, kf = to_f32(q).astype(np.float64), to_f32(k).astype(np.float64)
    for t in range(q_len):
        vis = kv_len - q_len + t + 1
        for h in range(hq):
            logits = scale * kf[:vis, h // (hq // hkv)] @ qf[t, h]
            p = softmax(logits)
            np.testing.assert_allclose(out[t, h, :vis], p, rtol=1e-12, atol=1e-15)
            assert np.all(out[t, h, vis:] == 0.0)          # causal inside the block
            np.testing.assert_allclose(out[t, h].sum(), 1.0, rtol=1e-13)
            np.testing.assert_allclose(lse[t, h], np.log(np.exp(logits).sum()), rtol=1e-12)


def test_gqa_head_mapping_uses_consecutive_groups():
    # kv head g carries value g+1 everywhere: q head h must return (h // G) + 1.
    hq, hkv, d = 8, 4, 8
    q, k = rnd((1, hq, d), 8), rnd((5, hkv, d), 9)
    v = np.zeros((5, hkv, d), np.float32)
    for g in range(hkv):
        v[:, g, :] = g + 1
    out, _ = oracle.decode_attn(q, k, to_bf16(v), 0.2)
    for h in range(hq):
        np.testing.assert_allclose(out[0, h], h // 2 + 1, rtol=1e-14)


def test_verify_rows_equal_truncated_single_query_calls():
    q_len, hq, hkv, d, kv_len = 5, 4, 2, 16, 61
    q, k, v = rnd((q_len, hq, d), 10), rnd((kv_len, hkv, d), 11), rnd((kv_len, hkv, d), 12)
    out, lse = oracle.decode_attn(q, k, v, 0.25)
    for t in range(q_len):
        vis = kv_len - q_len + t + 1
        o1, l1 = oracle.decode_attn(q[t:t + 1], k[:vis], v[:vis], 0.25)
        np.testing.assert_array_equal(out[t], o1[0])
        np.testing.assert_array_equal(lse[t], l1[0])


def test_permuting_past_keys_with_values_changes_nothing():
    hq, hkv, d, kv_len = 4, 1, 16, 50
    q, k, v = rnd((1, hq, d), 13), rnd((kv_len, hkv, d), 14), rnd((kv_len, hkv, d), 15)
    perm = np.random.default_rng(16).permutation(kv_len)
    a, la = oracle.decode_attn(q, k, v, 0.25)
    b, lb = oracle.decode_attn(q, k[perm], v[perm], 0.25)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(la, lb, rtol=1e-13)


def test_split_merge_identity():
    # flash-decode merge: o = sum_s e^{lse_s} o_s / sum_s e^{lse_s}; checked on
    # the oracle's own outputs over disjoint key ranges (q_len = 1).
    hq, hkv, d, kv_len = 2, 1, 8, 90
    q, k, v = rnd((1, hq, d), 17), rnd((kv_len, hkv, d), 18), rnd((kv_len, hkv, d), 19)
    full, lse = oracle.decode_attn(q, k, v, 0.35)
    parts = [oracle.decode_attn(q, k[a:b], v[a:b], 0.35) for a, b in ((0, 31), (31, 64), (64, 90))]
    w = np.stack([np.exp(l - lse) for _, l in parts])        # [3,1,hq]
    merged = sum(w[i][..., None] * parts[i][0] for i in range(3))
    np.testing.assert_allclose(w.sum(axis=0), 1.0, rtol=1e-12)
    np.testing.assert_allclose(merged, full, rtol=1e-11, atol=1e-14)


def test_scale_is_applied_to_logits_not_values():
    q, k, v = rnd((1, 1, 8), 20), rnd((9, 1, 8), 21), rnd((9, 1, 8), 22)
    out0, _ = oracle.decode_attn(q, k, v, 0.0)               # scale 0 -> uniform weights
    np.testing.assert_allclose(out0[0, 0], to_f32(v).astype(np.float64).mean(axis=0)[0], rtol=1e-13)


def test_rejects_bad_shapes():
    q, k = rnd((3, 3, 8), 23), rnd((2, 2, 8), 24)
    with pytest.raises(ValueError):
        oracle.decode_attn(q, k, k, 0.1)                      # q_len > kv_len, 3 % 2 != 0
