"""The seeded input generator: shapes, budgets, bf16 rounding, determinism."""
import numpy as np
import torch

from paper_2508_16201_amd import synth


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 10000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf], np.float32)])
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    back = synth.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_workload_sizes():
    sizes = {w.name: (w.n_video, w.keep_budget, w.k_top) for w in synth.WORKLOADS.values()}
    assert sizes["tiny"] == (1568, 157, 78)
    assert sizes["72b-1layer"] == (6272, 627, 313)
    assert sizes["72b-full"] == (12544, 1254, 627)
    assert sizes["32b-long"] == (32768, 3277, 1638)
    w = synth.V72B_FULL
    assert w.kv_len == 12544 + 256 + 6 and w.q_len == 6
    for pct, b in ((25, 8192), (50, 16384)):
        assert synth.scaled(synth.V32B_LONG, keep_percent=pct).keep_budget == b


def test_layer_is_deterministic_and_planted_keys_align():
    w = synth.TINY
    a, b = synth.make_layer(w), synth.make_layer(w)
    for key in a:
        np.testing.assert_array_equal(a[key], b[key])
    assert a["k"].shape == (w.kv_len, 1, 64) and a["q_text"].shape == (64, 4, 64)
    assert a["planted"].size == 32 and np.unique(a["planted"]).size == 32
    q = synth.bf16_bits_to_f32(a["q_text"]).astype(np.float64)
    k = synth.bf16_bits_to_f32(a["k"]).astype(np.float64)
    logit = [w.softmax_scale * q[i, :, :].mean(axis=0) @ k[j, 0] for j, i in zip(a["planted"], a["planted_query"])]
    np.testing.assert_allclose(logit, w.planted_logit, rtol=0.02)
    c = synth.make_layer(w, layer=1)
    assert not np.array_equal(a["k"], c["k"])


def test_ragged_lengths_in_range():
    f = synth.ragged_frames()
    assert f.shape == (8,) and f.min() >= 21 and f.max() <= 167
    assert 4096 <= f.min() * 196 and f.max() * 196 <= 32768


def test_accept_inputs():
    inp = synth.make_accept_inputs(2, 5, 100, 3, greedy=True)
    assert inp["target_logits"].shape == (2, 6, 100) and inp["draft_logits"].shape == (2, 5, 100)
    np.testing.assert_array_equal(inp["draft_tokens"], inp["draft_logits"].argmax(-1))
    assert inp["uniforms"].min() >= 0 and inp["uniforms"].max() < 1
