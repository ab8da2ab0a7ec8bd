"""GPU parity for the draft-tree variants: specvlm_tree_attn (ancestor mask
inside the verify block) and specvlm_accept_tree (greedy walk), against the
oracle."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2508_16201_amd import synth
from gpu_util import dev_bf16, host_f64, rnd_bits, assert_attn_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2508_16201_amd import binding
    binding.lib()
    return binding


def dev_mask(m):
    return torch.from_numpy(np.ascontiguousarray(m).view(np.int64)).cuda()


@pytest.mark.parametrize("n_nodes,kv_ctx,hq,hkv,d,splits,seed", [
    (7, 1632, 4, 1, 64, 0, 0),        # Tiny-shaped context, 7-node tree
    (8, 3000, 16, 2, 128, 0, 1),      # 64 rows per kv head
    (6, 6400, 64, 8, 128, 0, 2),      # 72B single-layer shape, 6 nodes
    (5, 40, 8, 2, 64, 1, 3),          # the block is a third of the cache
    (12, 500, 10, 2, 128, 3, 4),      # group 5, 60 rows
    (26, 2000, 2, 1, 128, 0, 5),      # a 26-node tree (EAGLE-sized), 2 q heads
    (26, 6400, 64, 8, 128, 0, 6),     # the same tree size at the 72B head shape: 208 rows per kv head
    (60, 3000, 64, 8, 128, 0, 7),     # 60 nodes at 64/8 heads: 480 rows per kv head, eight row groups
    (60, 2100, 28, 4, 128, 0, 8),     # 60 nodes at the 7B head shape (group 7): 420 rows
    (26, 2100, 28, 4, 128, 4, 9),
    (64, 500, 40, 8, 128, 0, 10),     # the largest tree the mask holds, 32B head shape (group 5)
])
def test_tree_attn_matches_oracle(B, n_nodes, kv_ctx, hq, hkv, d, splits, seed):
    parent = synth.make_tree(n_nodes, seed=40 + seed)
    masks = synth.ancestor_masks(parent)
    kv_len = kv_ctx + n_nodes
    q, k, v = rnd_bits((n_nodes, hq, d), 50 + seed), rnd_bits((kv_len, hkv, d), 60 + seed), rnd_bits((kv_len, hkv, d), 70 + seed)
    scale = 1 / np.sqrt(d)
    want, want_lse = oracle.tree_attn(q, k, v, masks, scale)
    out, lse = B.tree_attn(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, dev_mask(masks), want_lse=True,
                           num_splits=splits)
    torch.cuda.synchronize()
    assert_attn_close(out, want, f"tree {n_nodes} nodes")
    np.testing.assert_allclose(host_f64(lse), want_lse, atol=2e-3, rtol=1e-4)


def test_chain_mask_equals_decode_attn_bitwise(B):
    q, k, v = rnd_bits((6, 16, 128), 80), rnd_bits((2500, 2, 128), 81), rnd_bits((2500, 2, 128), 82)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    chain = synth.ancestor_masks([-1, 0, 1, 2, 3, 4])
    a = B.decode_attn(qd, kd, vd, 0.088, num_splits=5)
    b = B.tree_attn(qd, kd, vd, 0.088, dev_mask(chain), num_splits=5)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_tree_attn_ragged_batch_of_large_trees(B):
    """Trees of 26-60 nodes at 64/8 heads in one launch with cu arrays (more than 64 rows per kv head:
    uniform key splits, several row groups per head)."""
    hq, hkv, d = 64, 8, 128
    trees = [synth.make_tree(n, seed=190 + i) for i, n in enumerate((26, 60, 9))]
    lens = [900 + 26, 64 + 60, 2300 + 9]
    qs = [rnd_bits((t.size, hq, d), 200 + i) for i, t in enumerate(trees)]
    ks = [rnd_bits((n, hkv, d), 210 + i) for i, n in enumerate(lens)]
    vs = [rnd_bits((n, hkv, d), 220 + i) for i, n in enumerate(lens)]
    masks = [synth.ancestor_masks(t) for t in trees]
    cu_q = torch.tensor(np.concatenate([[0], np.cumsum([t.size for t in trees])]), dtype=torch.int32).cuda()
    cu_kv = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32).cuda()
    out = B.tree_attn(dev_bf16(np.concatenate(qs)), dev_bf16(np.concatenate(ks)), dev_bf16(np.concatenate(vs)),
                      0.088, dev_mask(np.concatenate(masks)), cu_q=cu_q, cu_kv=cu_kv,
                      max_q_len=60, max_kv_len=max(lens))
    torch.cuda.synchronize()
    o = 0
    for i, t in enumerate(trees):
        want, _ = oracle.tree_attn(qs[i], ks[i], vs[i], masks[i], 0.088)
        assert_attn_close(out[o:o + t.size], want, f"large tree, request {i}")
        o += t.size


def test_tree_attn_ragged_batch(B):
    hq, hkv, d = 8, 2, 128
    trees = [synth.make_tree(n, seed=90 + i) for i, n in enumerate((5, 9, 3))]
    lens = [700 + 5, 64 + 9, 1300 + 3]
    qs = [rnd_bits((t.size, hq, d), 100 + i) for i, t in enumerate(trees)]
    ks = [rnd_bits((n, hkv, d), 110 + i) for i, n in enumerate(lens)]
    vs = [rnd_bits((n, hkv, d), 120 + i) for i, n in enumerate(lens)]
    masks = [synth.ancestor_masks(t) for t in trees]
    cu_q = torch.tensor(np.concatenate([[0], np.cumsum([t.size for t in trees])]), dtype=torch.int32).cuda()
    cu_kv = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32).cuda()
    out = B.tree_attn(dev_bf16(np.concatenate(qs)), dev_bf16(np.concatenate(ks)), dev_bf16(np.concatenate(vs)),
                      0.088, dev_mask(np.concatenate(masks)), cu_q=cu_q, cu_kv=cu_kv, max_q_len=9,
                      max_kv_len=max(lens))
    torch.cuda.synchronize()
    o = 0
    for i, t in enumerate(trees):
        want, _ = oracle.tree_attn(qs[i], ks[i], vs[i], masks[i], 0.088)
        assert_attn_close(out[o:o + t.size], want, f"ragged tree {i}")
        o += t.size


def test_accept_tree_golden_walks(B):
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tree_traces.json")))
    parent = torch.tensor(g["parent"], dtype=torch.int32).cuda()
    traces = g["traces"]
    logits = np.zeros((len(traces), 7, 10), np.float32)
    tokens = np.zeros((len(traces), 7), np.int32)
    for b, tr in enumerate(traces):
        for i, t in enumerate(tr["target_argmax"]):
            logits[b, i, t] = 1.0
        tokens[b] = tr["tokens"]
    n, nodes, out = B.accept_tree(torch.from_numpy(logits).cuda(), torch.from_numpy(tokens).cuda(), parent)
    torch.cuda.synchronize()
    for b, tr in enumerate(traces):
        k = tr["n"]
        assert n[b].item() == k, tr["name"]
        assert nodes[b, :k].cpu().tolist() == tr["nodes"], tr["name"]
        assert out[b, :k + 1].cpu().tolist() == tr["out"], tr["name"]
        assert bool((nodes[b, k:] == -1).all()) and bool((out[b, k + 1:] == -1).all())


@pytest.mark.parametrize("batch,n_nodes,vocab", [(4, 26, 152064), (8, 7, 1024), (2, 64, 5000), (3, 1, 100)])
def test_accept_tree_bit_exact_on_random_trees(B, batch, n_nodes, vocab):
    parent = synth.make_tree(n_nodes, seed=130 + n_nodes)
    rng = np.random.default_rng(131 + n_nodes)
    logits = (3 * rng.standard_normal((batch, n_nodes, vocab))).astype(np.float32)
    # draft tokens: each node's children carry the parent's target token, a runner-up or a random
    # token, so walks of several lengths occur
    top2 = np.argsort(logits, axis=-1)[..., -2:]
    tokens = rng.integers(0, vocab, size=(batch, n_nodes)).astype(np.int32)
    for b in range(batch):
        for c in range(1, n_nodes):
            pick = rng.random()
            if pick < 0.6:
                tokens[b, c] = top2[b, parent[c], 1]
            elif pick < 0.8:
                tokens[b, c] = top2[b, parent[c], 0]
    n, nodes, out = B.accept_tree(torch.from_numpy(logits).cuda(), torch.from_numpy(tokens).cuda(),
                                  torch.from_numpy(parent).cuda())
    torch.cuda.synchronize()
    lengths = []
    for b in range(batch):
        wn, wnodes, wout = oracle.accept_tree_greedy(logits[b], tokens[b], parent)
        assert n[b].item() == wn
        np.testing.assert_array_equal(nodes[b].cpu().numpy(), wnodes)
        np.testing.assert_array_equal(out[b].cpu().numpy(), wout)
        lengths.append(wn)
    if n_nodes >= 7:
        assert max(lengths) >= 1


def test_tree_argument_errors(B):
    q = torch.zeros((3, 4, 64), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((10, 1, 64), dtype=torch.bfloat16, device="cuda")
    lib = B.lib()
    rc = lib.specvlm_tree_attn(q.data_ptr(), 256, 64, k.data_ptr(), k.data_ptr(), 64, 64, None, None, 1, 3, 10,
                               4, 1, 64, 0.1, None, q.data_ptr(), None, 0, None, 0, None)
    assert rc == -1                                         # mask missing
    t = torch.zeros((1, 70, 8), device="cuda")
    with pytest.raises(B.SpecVLMError) as e:
        B.accept_tree(t, torch.zeros((1, 70), dtype=torch.int32, device="cuda"),
                      torch.zeros(70, dtype=torch.int32, device="cuda"))
    assert e.value.status == -2
