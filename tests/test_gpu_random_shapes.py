"""GPU parity on seeded random shapes: every entry point of the path against the oracle on shapes drawn
inside the documented limits (head counts of the paper's models, both head sizes, split counts, ragged
batches), beyond the hand-picked cases of the other files.  Same bars as there: attention max-abs 2e-2 /
mean-abs 2e-3, scores 2e-3 relative, index and byte work bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_16201_amd import synth
from gpu_util import dev_bf16, host_f64, host_bits, rnd_bits, assert_attn_close

pytestmark = pytest.mark.gpu

HEADS = [(4, 1), (8, 2), (14, 2), (16, 2), (28, 4), (40, 8), (64, 8), (2, 2), (7, 1)]


@pytest.fixture(scope="module")
def B():
    from paper_2508_16201_amd import binding
    binding.lib()
    return binding


def i32(a):
    return torch.tensor(np.asarray(a, dtype=np.int32)).cuda()


def test_attention_chain_blocks(B):
    rng = np.random.default_rng(1101)
    for it in range(24):
        hq, hkv = HEADS[rng.integers(len(HEADS))]
        d = int(rng.choice([64, 128]))
        group = hq // hkv
        q_len = int(rng.integers(1, min(64, max(2, 300 // group)) + 1))      # up to ~300 rows per kv head
        kv_len = int(rng.integers(q_len, 5000))
        splits = int(rng.choice([0, 0, 1, 2, 3, 7, 13]))
        head_major = bool(rng.integers(2))
        seed = int(rng.integers(1 << 30))
        tag = f"case {it}: q{q_len} kv{kv_len} h{hq}/{hkv} d{d} splits{splits} head_major{head_major}"
        q, k, v = rnd_bits((q_len, hq, d), seed), rnd_bits((kv_len, hkv, d), seed + 1), rnd_bits((kv_len, hkv, d), seed + 2)
        scale = 1 / np.sqrt(d)
        want, want_lse = oracle.decode_attn(q, k, v, scale)
        kd, vd = dev_bf16(k), dev_bf16(v)
        if head_major:
            kd = kd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
            vd = vd.permute(1, 0, 2).contiguous().permute(1, 0, 2)
        out, lse = B.decode_attn(dev_bf16(q), kd, vd, scale, want_lse=True, num_splits=splits)
        torch.cuda.synchronize()
        assert_attn_close(out, want, tag)
        np.testing.assert_allclose(host_f64(lse), want_lse, atol=2e-3, rtol=1e-4, err_msg=tag)


def test_attention_trees(B):
    rng = np.random.default_rng(1102)
    for it in range(10):
        hq, hkv = HEADS[rng.integers(len(HEADS))]
        d = int(rng.choice([64, 128]))
        n_nodes = int(rng.integers(1, 65))
        kv_len = int(rng.integers(n_nodes, 3000))
        seed = int(rng.integers(1 << 30))
        parent = [-1] + [int(rng.integers(0, i)) for i in range(1, n_nodes)]
        mask = np.zeros(n_nodes, dtype=np.uint64)
        for i in range(n_nodes):
            m, j = 1 << i, parent[i]
            while j >= 0:
                m |= 1 << j
                j = parent[j]
            mask[i] = m
        q, k, v = rnd_bits((n_nodes, hq, d), seed), rnd_bits((kv_len, hkv, d), seed + 1), rnd_bits((kv_len, hkv, d), seed + 2)
        scale = 1 / np.sqrt(d)
        want, _ = oracle.tree_attn(q, k, v, mask, scale)
        out = B.tree_attn(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, torch.from_numpy(mask.view(np.int64)).cuda())
        torch.cuda.synchronize()
        assert_attn_close(out, want, f"case {it}: nodes{n_nodes} kv{kv_len} h{hq}/{hkv} d{d}")


def test_attention_ragged_batches(B):
    rng = np.random.default_rng(1103)
    for it in range(10):
        hq, hkv = HEADS[rng.integers(len(HEADS) - 1)]
        d = int(rng.choice([64, 128]))
        group = hq // hkv
        nb = int(rng.integers(2, 12))
        max_q = int(rng.integers(1, min(64, max(2, 128 // group)) + 1))
        q_lens = [int(rng.integers(1, max_q + 1)) for _ in range(nb)]
        lens = [int(rng.integers(q, int(rng.choice([300, 3000, 9000])))) for q in q_lens]
        splits = int(rng.choice([0, 0, 0, 1, 3]))
        seed = int(rng.integers(1 << 30))
        qs = [rnd_bits((ql, hq, d), seed + 3 * i) for i, ql in enumerate(q_lens)]
        ks = [rnd_bits((n, hkv, d), seed + 3 * i + 1) for i, n in enumerate(lens)]
        vs = [rnd_bits((n, hkv, d), seed + 3 * i + 2) for i, n in enumerate(lens)]
        scale = 1 / np.sqrt(d)
        out, lse = B.decode_attn(dev_bf16(np.concatenate(qs)), dev_bf16(np.concatenate(ks)),
                                 dev_bf16(np.concatenate(vs)), scale,
                                 cu_q=i32(np.concatenate([[0], np.cumsum(q_lens)])),
                                 cu_kv=i32(np.concatenate([[0], np.cumsum(lens)])), max_q_len=max(q_lens),
                                 max_kv_len=max(lens), want_lse=True, num_splits=splits)
        torch.cuda.synchronize()
        o = 0
        for i in range(nb):
            tag = f"case {it} request {i}: h{hq}/{hkv} d{d} q{q_lens[i]} kv{lens[i]} splits{splits}"
            want, want_lse = oracle.decode_attn(qs[i], ks[i], vs[i], scale)
            assert_attn_close(out[o:o + q_lens[i]], want, tag)
            np.testing.assert_allclose(host_f64(lse[o:o + q_lens[i]]), want_lse, atol=2e-3, rtol=1e-4, err_msg=tag)
            o += q_lens[i]


def test_scores_over_layers(B):
    rng = np.random.default_rng(1104)
    for it in range(10):
        hq, hkv = HEADS[rng.integers(len(HEADS))]
        d = int(rng.choice([64, 128]))
        V, L, P = int(rng.integers(1, 2500)), int(rng.integers(1, 200)), int(rng.integers(0, 20))
        mode, layers = int(rng.integers(2)), int(rng.integers(1, 4))
        # one case in four puts the first text queries inside the video span (causal columns)
        pos0 = P + V - int(rng.integers(0, min(V, 40))) if rng.integers(4) == 0 else P + V
        n_keys = max(pos0 + L, P + V)
        seed = int(rng.integers(1 << 30))
        qs = [rnd_bits((L, hq, d), seed + 10 * l) for l in range(layers)]
        ks = [rnd_bits((n_keys, hkv, d), seed + 10 * l + 1) for l in range(layers)]
        scale = 1 / np.sqrt(d)
        want = sum(oracle.score(q, k, P, V, pos0, scale, norm_mode=mode) for q, k in zip(qs, ks))
        got = B.score_layers(torch.stack([dev_bf16(q) for q in qs]), torch.stack([dev_bf16(k) for k in ks]), P, V,
                             pos0, scale, norm_mode=mode)
        torch.cuda.synchronize()
        g = host_f64(got)
        tag = f"case {it}: V{V} L{L} P{P} h{hq}/{hkv} d{d} mode{mode} layers{layers} pos0 {pos0}"
        assert np.isfinite(g).all(), tag
        assert (np.abs(g - want) <= 2e-3 * np.abs(want) + 1e-9).all(), (tag, float(np.abs(g - want).max()))


def random_scores(rng, n):
    kind = int(rng.integers(4))
    if kind == 0:
        s = synth.make_scores(n, int(rng.integers(1 << 20)))                     # long-tailed
    elif kind == 1:
        s = rng.integers(0, 8, n).astype(np.float32) / 8                         # eight levels: heavy ties
    elif kind == 2:
        s = ((1.0 + rng.standard_normal(n) * 1e-3) * 6e-3).astype(np.float32)    # a narrow band, as layer sums are
    else:
        s = rng.standard_normal(n).astype(np.float32)                            # signs, NaN, -0
        s[rng.integers(0, n, max(1, n // 50))] = np.nan
        s[rng.integers(0, n, max(1, n // 50))] = -0.0
    return np.ascontiguousarray(s, dtype=np.float32)


def test_select_single_requests(B):
    rng = np.random.default_rng(1105)
    for it in range(24):
        n = int(rng.integers(1, 65537)) if rng.integers(3) else int(rng.integers(1, 3000))
        budget = int(rng.integers(0, n + 1))
        k = int(rng.integers(0, budget + 1))
        s = random_scores(rng, n)
        wk, wf = oracle.select(s, k, budget)
        gk, gf = B.select(torch.from_numpy(s).cuda(), i32([k]), i32([budget]), budget)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(gk.cpu().numpy(), wk, err_msg=f"case {it}: n{n} k{k} budget{budget}")
        np.testing.assert_array_equal(gf.cpu().numpy(), wf, err_msg=f"case {it}: n{n} k{k} budget{budget}")


def test_select_ragged_batches(B):
    rng = np.random.default_rng(1106)
    for it in range(10):
        nb = int(rng.integers(1, 10))
        Vs = [int(rng.integers(1, int(rng.choice([500, 20000, 65536])))) for _ in range(nb)]
        buds = [int(rng.integers(0, v + 1)) for v in Vs]
        kts = [int(rng.integers(0, b + 1)) for b in buds]
        scores = [random_scores(rng, v) for v in Vs]
        keep, flag, status = B.select(torch.from_numpy(np.concatenate(scores)).cuda(), i32(kts), i32(buds),
                                      int(sum(buds)), cu_video=i32(np.concatenate([[0], np.cumsum(Vs)])),
                                      cu_keep=i32(np.concatenate([[0], np.cumsum(buds)])), max_n_video=max(Vs),
                                      want_status=True)
        torch.cuda.synchronize()
        assert status.cpu().numpy().tolist() == [0] * nb
        keep, flag = keep.cpu().numpy(), flag.cpu().numpy()
        o = 0
        for i in range(nb):
            wk, wf = oracle.select(scores[i], kts[i], buds[i])
            np.testing.assert_array_equal(keep[o:o + buds[i]], wk, err_msg=f"case {it} request {i}")
            np.testing.assert_array_equal(flag[o:o + buds[i]], wf, err_msg=f"case {it} request {i}")
            o += buds[i]


def test_top_p_counts(B):
    """Eq. 6's count on random sizes, score shapes (long-tailed, tied, a narrow band, signs / NaN / -0) and
    mass fractions; equality with the oracle wherever lambda * total is further than 1e-6 * total from a
    deciding prefix sum, at most one apart inside that margin."""
    rng = np.random.default_rng(1109)
    checked = 0
    for it in range(24):
        n = int(rng.integers(1, 65537)) if rng.integers(3) else int(rng.integers(1, 3000))
        s = random_scores(rng, n)
        lam = float(np.float32(rng.choice([0.02, 0.1, 0.3, 0.5, 0.8, 0.97])))
        want, margin = oracle.top_p_count(s, lam, want_margin=True)
        got = B.top_p_count(torch.from_numpy(s).cuda(), lam).item()
        torch.cuda.synchronize()
        if margin > 1e-6:
            assert got == want, (it, n, lam, got, want, margin)
            checked += 1
        else:
            assert abs(got - want) <= 1, (it, n, lam, got, want, margin)
    assert checked >= 12


def test_gather_rows(B):
    rng = np.random.default_rng(1107)
    for it in range(10):
        hkv, d, layers = int(rng.choice([1, 2, 4, 8, 3])), int(rng.choice([64, 128])), int(rng.integers(1, 4))
        V, P, T = int(rng.integers(1, 3000)), int(rng.integers(0, 10)), int(rng.integers(0, 100))
        keep = np.sort(rng.choice(V, int(rng.integers(0, V + 1)), replace=False)).astype(np.int32)
        seed = int(rng.integers(1 << 30))
        k, v = rnd_bits((layers, P + V + T, hkv, d), seed), rnd_bits((layers, P + V + T, hkv, d), seed + 1)
        kd, vd = B.gather_kv(dev_bf16(k), dev_bf16(v), P, V, torch.from_numpy(keep).cuda())
        torch.cuda.synchronize()
        for l in range(layers):
            tag = f"case {it} layer {l}: V{V} P{P} T{T} keep{keep.size} hkv{hkv} d{d}"
            np.testing.assert_array_equal(host_bits(kd[l]), oracle.gather_kv(k[l], P, V, keep), err_msg=tag)
            np.testing.assert_array_equal(host_bits(vd[l]), oracle.gather_kv(v[l], P, V, keep), err_msg=tag)


def test_greedy_accept(B):
    rng = np.random.default_rng(1108)
    for it in range(10):
        gamma, vocab = int(rng.integers(0, 20)), int(rng.choice([17, 1000, 8192, 8193, 32000, 152064]))
        batch = int(rng.integers(1, 5))
        acc = synth.make_accept_inputs(batch, gamma, vocab, int(rng.integers(1 << 20)))
        n, out = B.accept(torch.from_numpy(acc["target_logits"]).cuda(), torch.from_numpy(acc["draft_tokens"]).cuda())
        torch.cuda.synchronize()
        for b in range(batch):
            rn, rout = oracle.accept_greedy(acc["target_logits"][b], acc["draft_tokens"][b])
            tag = f"case {it} request {b}: gamma{gamma} vocab{vocab}"
            assert int(n[b]) == rn, tag
            assert out[b].cpu().tolist()[:rn + 1] == rout.tolist()[:rn + 1], tag
