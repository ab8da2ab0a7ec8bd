"""Seeded synthetic inputs for the SpecVLM hot path.

This module only *draws data*: shapes, value distributions and structure of a
video-LLM KV cache (frames x per-frame token grid, then a language prompt),
planted high-attention video keys, logits for the acceptance step.  It holds
none of the method's arithmetic (no softmax, no selection, no attention) and
imports neither the HIP binding nor the CPU oracle, so both can consume the
same arrays.

bf16 tensors are carried as ``uint16`` bit patterns (NumPy has no bf16); the
rounding helper below is plain round-to-nearest-even of an fp32 value to its
upper 16 bits.

Workload shapes follow the paper's experimental set-up (App. A: 196 tokens
per frame, 64 or 128 sampled frames; Sec. 3.2: long-tailed language-to-video
attention; default pruning ratio 90 %).  The paper's datasets and weights are
not available, so every value is synthetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np

SEED_BASE = 20250816


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (data plumbing only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One cache shape.  Token order in the cache: video (frame-major, then
    row-major on the frame's grid), then text, then the verify block."""
    name: str
    n_frames: int
    grid_h: int
    grid_w: int
    n_text: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_layers: int = 1
    gamma: int = 5
    keep_percent: int = 10
    vocab: int = 1024
    n_planted: int = 0            # 0 -> 2 % of the video tokens
    planted_logit: float = 11.0   # group-mean logit of a planted (query, key) pair
    # draft model cache shape (heads) for the decode loop over the pruned cache
    draft_q_heads: int = 0
    draft_kv_heads: int = 0
    draft_head_dim: int = 0
    draft_layers: int = 0
    index: int = 0                # position in the configuration list (seed offset)

    @property
    def n_video(self) -> int:
        return self.n_frames * self.grid_h * self.grid_w

    @property
    def n_ctx(self) -> int:
        """Keys before the verify block: video + text."""
        return self.n_video + self.n_text

    @property
    def q_len(self) -> int:
        return self.gamma + 1

    @property
    def kv_len(self) -> int:
        """Keys visible to the last query of the verify block."""
        return self.n_ctx + self.q_len

    @property
    def keep_budget(self) -> int:
        return (self.n_video * self.keep_percent + 50) // 100

    @property
    def k_top(self) -> int:
        return self.keep_budget // 2

    @property
    def planted(self) -> int:
        return self.n_planted if self.n_planted > 0 else (self.n_video * 2 + 50) // 100

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


TINY = Workload("tiny", 8, 14, 14, 64, 4, 1, 64, n_layers=1, gamma=4, vocab=1024,
                n_planted=32, draft_q_heads=4, draft_kv_heads=1, draft_head_dim=64,
                draft_layers=1, index=0)
V72B_1L = Workload("72b-1layer", 32, 14, 14, 128, 64, 8, 128, n_layers=1, gamma=5,
                   vocab=152064, draft_q_heads=64, draft_kv_heads=8, draft_head_dim=128,
                   draft_layers=1, index=1)
V72B_FULL = Workload("72b-full", 64, 14, 14, 256, 64, 8, 128, n_layers=80, gamma=5,
                     vocab=152064, draft_q_heads=14, draft_kv_heads=2, draft_head_dim=64,
                     draft_layers=24, index=2)
V32B_LONG = Workload("32b-long", 128, 16, 16, 256, 40, 8, 128, n_layers=64, gamma=5,
                     vocab=152064, draft_q_heads=28, draft_kv_heads=4, draft_head_dim=128,
                     draft_layers=28, index=3)
RAGGED = Workload("ragged-x8", 0, 14, 14, 256, 64, 8, 128, n_layers=1, gamma=5,
                  vocab=152064, draft_q_heads=28, draft_kv_heads=4, draft_head_dim=128,
                  draft_layers=1, index=4)
# Self-speculation with the 7B model (Sec. 4.1: 128 frames of 196 tokens): the draft is the verifier's
# own weights over the pruned cache, so both caches have the 28/4-head, 28-layer shape.
V7B_SELF = Workload("7b-self", 128, 14, 14, 256, 28, 4, 128, n_layers=28, gamma=5,
                    vocab=152064, draft_q_heads=28, draft_kv_heads=4, draft_head_dim=128,
                    draft_layers=28, index=5)

WORKLOADS: Dict[str, Workload] = {w.name: w for w in
                                  (TINY, V72B_1L, V72B_FULL, V32B_LONG, RAGGED, V7B_SELF)}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller test shapes)."""
    return replace(w, **kw)


def ragged_frames(batch: int = 8, seed: int = SEED_BASE + 4000) -> np.ndarray:
    """Per-request frame counts, uniform in {21..167}: with 196 tokens per
    frame the video lengths land in [4116, 32732]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(21, 168, size=batch).astype(np.int64)


# --------------------------------------------------------------------------
# Cache generator
# --------------------------------------------------------------------------
def layer_seed(w: Workload, layer: int, salt: int = 0) -> int:
    return SEED_BASE + 1000 * w.index + layer + 7919 * salt


def make_layer(w: Workload, layer: int = 0, *, n_q_heads: Optional[int] = None,
               n_kv_heads: Optional[int] = None, head_dim: Optional[int] = None,
               salt: int = 0, plant: bool = True) -> Dict[str, np.ndarray]:
    """One layer's tensors, all bf16 bit patterns (uint16):

      q_text  [n_text, H_q, d]     queries of the language prompt
      k, v    [kv_len, H_kv, d]    video rows, text rows, then the verify block's rows
      q_block [gamma+1, H_q, d]    queries of the verify block
      planted [n_planted] int64    video-local indices of the planted keys
      planted_query [n_planted]    text query each planted key is aligned to

    Q, K, V are i.i.d. N(0,1).  A planted key j paired with text query i* is
    overwritten, for every kv head g, by  c * qbar/|qbar|  where qbar is the
    mean of Q[i*, h, :] over the q heads h of group g and c is chosen so that
    the group-mean scaled logit of the pair equals ``planted_logit``.
    """
    hq = n_q_heads or w.n_q_heads
    hkv = n_kv_heads or w.n_kv_heads
    d = head_dim or w.head_dim
    group = hq // hkv
    rng = np.random.Generator(np.random.PCG64(layer_seed(w, layer, salt)))
    q_text = rng.standard_normal((w.n_text, hq, d), dtype=np.float32)
    k = rng.standard_normal((w.kv_len, hkv, d), dtype=np.float32)
    v = rng.standard_normal((w.kv_len, hkv, d), dtype=np.float32)
    q_block = rng.standard_normal((w.q_len, hq, d), dtype=np.float32)
    n_p = min(w.planted, w.n_video) if plant else 0
    planted = np.sort(rng.choice(w.n_video, size=n_p, replace=False)) if n_p else \
        np.zeros(0, dtype=np.int64)
    planted_query = rng.integers(0, max(w.n_text, 1), size=n_p)
    if n_p:
        scale = 1.0 / np.sqrt(d)
        # the queries are what the kernels will see: round them first
        q_seen = bf16_bits_to_f32(f32_to_bf16_bits(q_text))
        qbar = q_seen[planted_query].reshape(n_p, hkv, group, d).mean(axis=2)
        norm = np.linalg.norm(qbar, axis=-1, keepdims=True)
        c = w.planted_logit / (scale * norm)
        k[planted] = (c * qbar / norm).astype(np.float32)
    return {
        "q_text": f32_to_bf16_bits(q_text),
        "k": f32_to_bf16_bits(k),
        "v": f32_to_bf16_bits(v),
        "q_block": f32_to_bf16_bits(q_block),
        "planted": planted.astype(np.int64),
        "planted_query": planted_query.astype(np.int64),
    }


def make_scores(n_video: int, seed: int, *, levels: int = 0, heavy_frac: float = 0.02
                ) -> np.ndarray:
    """A long-tailed fp32 score vector for selection tests: a flat background
    near 1/n with a few heavy entries.  ``levels`` > 0 quantises the values to
    that many distinct levels (duplicate-score stress)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    base = (1.0 + 0.05 * rng.standard_normal(n_video)) / max(n_video, 1)
    n_heavy = int(round(heavy_frac * n_video))
    if n_heavy:
        idx = rng.choice(n_video, size=n_heavy, replace=False)
        base[idx] *= 20.0 + 80.0 * rng.random(n_heavy)
    s = np.abs(base).astype(np.float32)
    if levels > 0 and n_video:
        lo, hi = float(s.min()), float(s.max())
        q = np.floor((s - lo) / max(hi - lo, 1e-30) * (levels - 1) + 0.5)
        s = (lo + q * (hi - lo) / max(levels - 1, 1)).astype(np.float32)
    return s


# --------------------------------------------------------------------------
# Acceptance inputs
# --------------------------------------------------------------------------
def make_accept_inputs(batch: int, gamma: int, vocab: int, seed: int, *,
                       sigma: float = 0.3, greedy: bool = True,
                       temperature: float = 1.0) -> Dict[str, np.ndarray]:
    """Target logits ~ 3 N(0,1); draft logits = target + sigma N(0,1) (sigma 0.3:
    the draft's argmax equals the target's about 80 % of the time, i.e. about 3.7
    tokens per step at gamma 5, the regime of the paper's tau = 3.48).
    Draft tokens are the draft row's argmax (greedy) or drawn from the draft's
    own distribution with the generator (sampling).  Uniforms in [0,1) fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    target = (3.0 * rng.standard_normal((batch, gamma + 1, vocab))).astype(np.float32)
    draft = (target[:, :gamma, :] +
             sigma * rng.standard_normal((batch, gamma, vocab))).astype(np.float32)
    if greedy:
        tokens = draft.argmax(axis=-1).astype(np.int32) if gamma else \
            np.zeros((batch, 0), dtype=np.int32)
    else:
        # Gumbel-max draw from the draft rows: a data draw, independent of the
        # acceptance rule under test.
        g = -np.log(-np.log(rng.random((batch, gamma, vocab)) * (1 - 1e-12) + 1e-12))
        tokens = (draft.astype(np.float64) / temperature + g).argmax(axis=-1).astype(np.int32) \
            if gamma else np.zeros((batch, 0), dtype=np.int32)
    u = rng.random((batch, gamma + 1), dtype=np.float32)
    u = np.minimum(u, np.float32(1.0 - 2.0 ** -24)).astype(np.float32)
    return {"target_logits": target, "draft_logits": draft,
            "draft_tokens": tokens.reshape(batch, gamma), "uniforms": u}


# --------------------------------------------------------------------------
# Draft trees (structure only)
# --------------------------------------------------------------------------
def ancestor_masks(parent) -> np.ndarray:
    """uint64 mask per node: bit b set iff b is the node itself or one of its ancestors."""
    parent = np.asarray(parent, dtype=np.int64)
    n = parent.shape[0]
    masks = np.zeros(n, dtype=np.uint64)
    for i in range(n):
        m, j = 0, i
        while j >= 0:
            m |= 1 << int(j)
            j = int(parent[j])
        masks[i] = np.uint64(m)
    return masks


def make_tree(n_nodes: int, seed: int, max_children: int = 3) -> np.ndarray:
    """A random static draft tree: parent[0] = -1, parent[i] < i, bounded fan-out."""
    rng = np.random.Generator(np.random.PCG64(seed))
    parent = np.full(n_nodes, -1, dtype=np.int32)
    fan = np.zeros(n_nodes, dtype=np.int64)
    for i in range(1, n_nodes):
        cand = [j for j in range(i) if fan[j] < max_children]
        j = int(rng.choice(cand))
        parent[i] = j
        fan[j] += 1
    return parent
