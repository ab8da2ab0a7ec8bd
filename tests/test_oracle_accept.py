"""Pins for the acceptance oracle: hand-enumerated greedy traces (golden file),
losslessness, special cases of the rejection-sampling rule, and a Monte-Carlo
check that the emitted token follows the target distribution."""
import json
import os

import numpy as np
import pytest
from scipy.special import softmax
from scipy.stats import chisquare

import oracle
from paper_2508_16201_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accept_traces.json")


def test_hand_enumerated_greedy_traces():
    traces = json.load(open(GOLDEN))["traces"]
    assert len(traces) >= 6
    for tr in traces:
        gamma, vocab = 4, 8
        logits = np.zeros((gamma + 1, vocab), np.float32)
        for i, t in enumerate(tr["target_argmax"]):
            logits[i, t] = 1.0
        for row, tok in tr.get("tie_with", {}).items():
            logits[int(row), tok] = 1.0
        n, out = oracle.accept_greedy(logits, np.array(tr["draft"], np.int32))
        assert n == tr["n"], tr["name"]
        np.testing.assert_array_equal(out, tr["out"], err_msg=tr["name"])


def test_greedy_is_lossless():
    # the emitted tokens are always a prefix of the target's own argmax chain
    for seed in range(20):
        inp = synth.make_accept_inputs(1, 5, 64, 100 + seed, sigma=1.5)
        t = inp["target_logits"][0]
        n, out = oracle.accept_greedy(t, inp["draft_tokens"][0])
        chain = t.argmax(axis=-1)
        np.testing.assert_array_equal(out[:n + 1], chain[:n + 1])
        assert np.all(out[n + 1:] == -1)
        if n < 5:
            assert inp["draft_tokens"][0][n] != chain[n]


def test_gamma_zero_is_plain_decoding():
    t = np.array([[0.1, 2.0, -1.0]], np.float32)
    n, out = oracle.accept_greedy(t, np.zeros(0, np.int32))
    assert n == 0 and list(out) == [1]
    n, out, _ = oracle.accept_sample(t, np.zeros((0, 3), np.float32), np.zeros(0, np.int32),
                                     np.array([0.0], np.float32))
    assert n == 0 and out[0] == 0              # u = 0 picks the first token with positive mass


def test_identical_models_accept_everything():
    inp = synth.make_accept_inputs(1, 6, 50, 7, sigma=0.0, greedy=False)
    for u0 in (0.0, 0.5, 0.999999):
        u = np.full(7, u0, np.float32)
        n, out, _ = oracle.accept_sample(inp["target_logits"][0], inp["draft_logits"][0],
                                         inp["draft_tokens"][0], u)
        assert n == 6
        np.testing.assert_array_equal(out[:6], inp["draft_tokens"][0])


def test_disjoint_one_hot_models_reject_at_once():
    vocab = 6
    t = np.full((3, vocab), -1e4, np.float32); t[:, 4] = 0.0        # target: all mass on 4
    dl = np.full((2, vocab), -1e4, np.float32); dl[:, 1] = 0.0      # draft: all mass on 1
    n, out, _ = oracle.accept_sample(t, dl, np.array([1, 1], np.int32),
                                     np.array([0.3, 0.3, 0.9], np.float32))
    assert n == 0 and out[0] == 4 and out[1] == -1


def test_zero_uniform_accepts_whatever_target_supports():
    inp = synth.make_accept_inputs(1, 4, 32, 8, sigma=2.0, greedy=False)
    u = np.zeros(5, np.float32)
    n, _, _ = oracle.accept_sample(inp["target_logits"][0], inp["draft_logits"][0],
                                   inp["draft_tokens"][0], u)
    assert n == 4


def test_threshold_and_residual_by_hand():
    # vocab 3, gamma 1.  p = (.5,.3,.2), q = (.2,.6,.2); x = 1: accept iff u*0.6 < 0.3.
    p = np.array([.5, .3, .2]); q = np.array([.2, .6, .2])
    t = np.log(np.stack([p, p])).astype(np.float32)
    dl = np.log(q)[None].astype(np.float32)
    x = np.array([1], np.int32)
    n, out, m = oracle.accept_sample(t, dl, x, np.array([0.49, 0.0], np.float32))
    assert n == 1 and out[0] == 1 and out[1] == 0
    n, out, m = oracle.accept_sample(t, dl, x, np.array([0.51, 0.99], np.float32))
    # rejected; residual max(p-q,0) = (.3, 0, 0) -> token 0 whatever the uniform
    assert n == 0 and list(out) == [0, -1]
    assert abs(m[0] - (0.51 * 0.6 - 0.3) / (0.51 * 0.6)) < 1e-6
    # bonus draw when everything is accepted uses p of the last row: cdf .5/.8/1
    for u1, tok in ((0.49, 0), (0.51, 1), (0.79, 1), (0.81, 2)):
        n, out, _ = oracle.accept_sample(t, dl, x, np.array([0.1, u1], np.float32))
        assert n == 1 and out[1] == tok


def test_final_token_interval_brackets_the_draw():
    p = np.array([.5, .3, .2]); q = np.array([.2, .6, .2])
    t = np.log(np.stack([p, p])).astype(np.float32)
    dl = np.log(q)[None].astype(np.float32)
    # after 1 accepted (bonus draw from p): cdf .5/.8/1
    for tok, (lo, hi) in enumerate(((0, .5), (.5, .8), (.8, 1.0))):
        a, b = oracle.final_token_interval(t, dl, 1, tok)
        assert abs(a - lo) < 1e-7 and abs(b - hi) < 1e-7
    # after a rejection at 0: residual (.3,0,0)/.3 -> token 0 owns [0,1)
    assert oracle.final_token_interval(t, dl, 0, 0) == pytest.approx((0.0, 1.0))
    a, b = oracle.final_token_interval(t, dl, 0, 2)
    assert a == pytest.approx(1.0) and b == pytest.approx(1.0)
    # consistent with the sampler on random inputs
    inp = synth.make_accept_inputs(1, 3, 200, 21, sigma=1.0, greedy=False)
    n, out, _ = oracle.accept_sample(inp["target_logits"][0], inp["draft_logits"][0],
                                     inp["draft_tokens"][0], inp["uniforms"][0])
    lo, hi = oracle.final_token_interval(inp["target_logits"][0], inp["draft_logits"][0], n, int(out[n]))
    assert lo <= inp["uniforms"][0][3] < hi


def test_temperature_scales_logits():
    p = np.array([.5, .3, .2]); q = np.array([.2, .6, .2])
    T = 2.0
    t = (T * np.log(np.stack([p, p]))).astype(np.float32)
    dl = (T * np.log(q))[None].astype(np.float32)
    n, _, _ = oracle.accept_sample(t, dl, np.array([1], np.int32), np.array([0.49, 0.0], np.float32), T)
    assert n == 1
    n, _, _ = oracle.accept_sample(t, dl, np.array([1], np.int32), np.array([0.51, 0.0], np.float32), T)
    assert n == 0


def test_monte_carlo_first_token_follows_target_distribution():
    """Distribution preservation: with x ~ q and fresh uniforms, the first
    emitted token is distributed as p_0 whatever q is."""
    vocab, gamma, trials = 16, 2, 200_000
    rng = np.random.default_rng(1234)
    t = (1.5 * rng.standard_normal((gamma + 1, vocab))).astype(np.float32)
    dl = (t[:gamma] + 1.2 * rng.standard_normal((gamma, vocab))).astype(np.float32)
    p0 = softmax(t[0].astype(np.float64))
    qs = [softmax(dl[i].astype(np.float64)) for i in range(gamma)]
    xs = np.stack([rng.choice(vocab, size=trials, p=qs[i]) for i in range(gamma)], axis=1).astype(np.int32)
    us = rng.random((trials, gamma + 1)).astype(np.float32)
    counts = np.zeros(vocab)
    n_hist = np.zeros(gamma + 1)
    for r in range(trials):
        n, out, _ = oracle.accept_sample(t, dl, xs[r], us[r])
        counts[out[0]] += 1
        n_hist[n] += 1
    stat, pval = chisquare(counts, p0 * trials)
    assert pval > 1e-3, (stat, pval)
    # acceptance rate of the first test is sum_v min(p, q)
    np.testing.assert_allclose(1 - n_hist[0] / trials, np.minimum(p0, qs[0]).sum(), atol=5e-3)


def test_rejects_bad_arguments():
    t = np.zeros((2, 4), np.float32); dl = np.zeros((1, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.accept_sample(t, dl, np.array([0], np.int32), np.zeros(2, np.float32), temperature=0.0)
    with pytest.raises(ValueError):
        oracle.accept_sample(t, dl, np.array([9], np.int32), np.zeros(2, np.float32))
