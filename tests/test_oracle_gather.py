"""Pins for the draft-cache gather oracle (end of Sec. 3.2: the draft keeps
V_R u V_U and the language prompt)."""
import numpy as np

import oracle
from paper_2508_16201_amd.synth import f32_to_bf16_bits as to_bf16, bf16_bits_to_f32 as to_f32


def rnd(shape, seed):
    return to_bf16(np.random.default_rng(seed).standard_normal(shape).astype(np.float32))


def test_matches_numpy_fancy_indexing():
    P, V, L = 3, 40, 5
    src = rnd((P + V + L, 2, 8), 0)
    keep = np.array([0, 3, 4, 17, 39], np.int32)
    dst = oracle.gather_kv(src, P, V, keep)
    rows = np.concatenate([np.arange(P), P + keep, np.arange(P + V, P + V + L)])
    np.testing.assert_array_equal(dst, src[rows])


def test_identity_and_empty():
    src = rnd((20, 1, 4), 1)
    np.testing.assert_array_equal(oracle.gather_kv(src, 2, 10, np.arange(10)), src)
    dst = oracle.gather_kv(src, 2, 10, np.zeros(0, np.int32))
    np.testing.assert_array_equal(dst, np.concatenate([src[:2], src[12:]]))


def test_attention_over_gathered_cache_equals_masked_attention():
    # dropping keys == giving them zero weight: compare with a library softmax
    # over the kept rows of the full cache.
    from scipy.special import softmax
    V, L, d = 30, 4, 16
    k, v, q = rnd((V + L, 1, d), 2), rnd((V + L, 1, d), 3), rnd((1, 2, d), 4)
    keep = np.array([1, 2, 9, 20, 29], np.int32)
    kg, vg = oracle.gather_kv(k, 0, V, keep), oracle.gather_kv(v, 0, V, keep)
    out, _ = oracle.decode_attn(q, kg, vg, 0.25)
    rows = np.concatenate([keep, np.arange(V, V + L)])
    kf, vf, qf = (to_f32(x).astype(np.float64) for x in (k, v, q))
    for h in range(2):
        p = softmax(0.25 * kf[rows, 0] @ qf[0, h])
        np.testing.assert_allclose(out[0, h], p @ vf[rows, 0], rtol=1e-12, atol=1e-15)
