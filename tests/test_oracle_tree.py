"""Pins for the tree-verification oracles (tree attention mask, greedy tree
acceptance): reduction to the chain case, branch isolation, hand traces."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2508_16201_amd import synth
from paper_2508_16201_amd.synth import f32_to_bf16_bits as to_bf16

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_traces.json")


def rnd(shape, seed):
    return to_bf16(np.random.default_rng(seed).standard_normal(shape).astype(np.float32))


def test_ancestor_masks():
    parent = [-1, 0, 0, 1, 1, 2, 3]
    m = synth.ancestor_masks(parent)
    assert [int(x) for x in m] == [0b1, 0b11, 0b101, 0b1011, 0b10011, 0b100101, 0b1001011]
    chain = synth.ancestor_masks([-1, 0, 1, 2])
    assert [int(x) for x in chain] == [1, 3, 7, 15]


def test_chain_mask_reproduces_causal_block():
    q, k, v = rnd((5, 4, 16), 0), rnd((70, 2, 16), 1), rnd((70, 2, 16), 2)
    chain = synth.ancestor_masks([-1, 0, 1, 2, 3])
    a, la = oracle.tree_attn(q, k, v, chain, 0.25)
    b, lb = oracle.decode_attn(q, k, v, 0.25)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(la, lb)


def test_each_node_equals_a_chain_over_its_root_path():
    """Node t's output must equal plain causal attention over the cache that
    holds the context followed by only t's ancestors (in order) and t itself."""
    parent = synth.make_tree(9, seed=3)
    masks = synth.ancestor_masks(parent)
    ctx, n, hq, hkv, d = 40, 9, 4, 2, 16
    q, k, v = rnd((n, hq, d), 4), rnd((ctx + n, hkv, d), 5), rnd((ctx + n, hkv, d), 6)
    out, lse = oracle.tree_attn(q, k, v, masks, 0.3)
    for t in range(n):
        path = [b for b in range(n) if (int(masks[t]) >> b) & 1]
        assert path[-1] == t
        rows = list(range(ctx)) + [ctx + b for b in path]
        o1, l1 = oracle.decode_attn(q[t:t + 1], k[rows], v[rows], 0.3)
        np.testing.assert_allclose(out[t], o1[0], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse[t], l1[0], rtol=1e-13)


def test_siblings_do_not_see_each_other():
    # two children of the root with very different values: each child's output
    # must ignore the other's value row
    ctx, d = 3, 8
    q = to_bf16(np.zeros((3, 1, d), np.float32))                 # uniform weights
    k = rnd((ctx + 3, 1, d), 7)
    v = np.zeros((ctx + 3, 1, d), np.float32)
    v[ctx + 1] = 100.0; v[ctx + 2] = -100.0
    masks = synth.ancestor_masks([-1, 0, 0])
    out, _ = oracle.tree_attn(q, k, to_bf16(v), masks, 0.5)
    np.testing.assert_allclose(out[1, 0], 100.0 / 5, rtol=1e-13)     # context(3) + root + itself
    np.testing.assert_allclose(out[2, 0], -100.0 / 5, rtol=1e-13)


def test_hand_enumerated_tree_walks():
    g = json.load(open(GOLDEN))
    parent = np.array(g["parent"], np.int32)
    for tr in g["traces"]:
        logits = np.zeros((7, 10), np.float32)
        for i, t in enumerate(tr["target_argmax"]):
            logits[i, t] = 1.0
        n, nodes, out = oracle.accept_tree_greedy(logits, np.array(tr["tokens"], np.int32), parent)
        assert n == tr["n"], tr["name"]
        assert nodes[:n].tolist() == tr["nodes"], tr["name"]
        assert out[:n + 1].tolist() == tr["out"], tr["name"]
        assert np.all(nodes[n:] == -1) and np.all(out[n + 1:] == -1)


def test_chain_tree_equals_chain_acceptance_and_is_lossless():
    for seed in range(10):
        inp = synth.make_accept_inputs(1, 5, 64, 900 + seed, sigma=0.8)
        t, x = inp["target_logits"][0], inp["draft_tokens"][0]
        n, out = oracle.accept_greedy(t, x)
        parent = np.array([-1, 0, 1, 2, 3, 4], np.int32)
        tokens = np.concatenate([[0], x]).astype(np.int32)
        tn, nodes, tout = oracle.accept_tree_greedy(t, tokens, parent)
        assert tn == n
        np.testing.assert_array_equal(tout[:n + 1], out[:n + 1])
        assert nodes[:n].tolist() == list(range(1, n + 1))
        # lossless: the emitted tokens follow the target's own argmax along the accepted path
        path = [0] + nodes[:n].tolist()
        for i, node in enumerate(path):
            assert tout[i] == t[node].argmax()


def test_rejects_bad_trees():
    logits = np.zeros((3, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.accept_tree_greedy(logits, np.zeros(3, np.int32), np.array([-1, 2, 0], np.int32))
