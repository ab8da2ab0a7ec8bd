"""ctypes front end of the CPU oracle (``specvlm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the benchmark's CPU-baseline leg, never by the product package.  The
wrapper only marshals NumPy arrays; every piece of arithmetic is in the C file.
bf16 tensors are ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specvlm_oracle.c")
_LIB = os.path.join(_HERE, "libspecvlm_oracle.so")
_lib = None


# SPECVLM_ORACLE_SANITIZE=1: an AddressSanitizer + UndefinedBehaviorSanitizer build of the same source
# (tests/test_oracle_sanitized.py runs the oracle's pins under it in a child process that preloads
# the sanitizer runtime).
_SANITIZE = os.environ.get("SPECVLM_ORACLE_SANITIZE") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libspecvlm_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 loops, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("oracle_decode_attn", "oracle_score", "oracle_select", "oracle_top_p_count",
                     "oracle_gather_kv", "oracle_accept_greedy", "oracle_accept_sample",
                     "oracle_final_token_interval", "oracle_tree_attn", "oracle_accept_tree_greedy"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def decode_attn(q, k, v, scale: float, want_lse: bool = True
                ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """q [q_len,H_q,d], k/v [kv_len,H_kv,d] (bf16 bits) -> out fp64 [q_len,H_q,d], lse [q_len,H_q]."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    q_len, hq, d = q.shape
    kv_len, hkv, _ = k.shape
    out = np.zeros((q_len, hq, d), dtype=np.float64)
    lse = np.zeros((q_len, hq), dtype=np.float64) if want_lse else None
    rc = lib().oracle_decode_attn(_p(q), _p(k), _p(v), q_len, kv_len, hq, hkv, d,
                                  C.c_double(scale), _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_decode_attn rc={rc}")
    return out, lse


def score(q_text, k, video_start: int, n_video: int, text_pos0: int, scale: float,
          norm_mode: int = 0, beta: float = 0.0, scores_in: Optional[np.ndarray] = None,
          want_lse: bool = False):
    """q_text [L,H_q,d], k [n_keys,H_kv,d] (bf16 bits) -> scores fp64 [n_video] (and row lse)."""
    q_text, k = _u16(q_text), _u16(k)
    n_text, hq, d = q_text.shape
    n_keys, hkv, _ = k.shape
    scores = np.zeros(n_video, dtype=np.float64) if scores_in is None else \
        np.array(scores_in, dtype=np.float64, copy=True)
    lse = np.zeros((n_text, hq), dtype=np.float64) if want_lse else None
    rc = lib().oracle_score(_p(q_text), _p(k), n_text, n_keys, video_start, n_video, text_pos0,
                            hq, hkv, d, C.c_double(scale), norm_mode, C.c_double(beta),
                            _p(scores), _p(lse))
    if rc:
        raise ValueError(f"oracle_score rc={rc}")
    return (scores, lse) if want_lse else scores


def select(scores, k_top: int, keep_budget: int) -> Tuple[np.ndarray, np.ndarray]:
    """fp32 scores [V] -> (keep_idx int32 [B] ascending, from_topk uint8 [B])."""
    s = np.ascontiguousarray(scores, dtype=np.float32)
    keep = np.zeros(max(keep_budget, 0), dtype=np.int32)
    flag = np.zeros(max(keep_budget, 0), dtype=np.uint8)
    rc = lib().oracle_select(_p(s), s.shape[0], k_top, keep_budget, _p(keep), _p(flag))
    if rc:
        raise ValueError(f"oracle_select rc={rc}")
    return keep, flag


def top_p_count(scores, lam: float, want_margin: bool = False):
    s = np.ascontiguousarray(scores, dtype=np.float32)
    margin = C.c_double(1.0)
    c = lib().oracle_top_p_count(_p(s), s.shape[0], C.c_double(lam), C.byref(margin))
    if c < 0:
        raise ValueError(f"oracle_top_p_count rc={c}")
    return (c, margin.value) if want_margin else c


def gather_kv(src, video_start: int, n_video: int, keep_idx) -> np.ndarray:
    """src [n_keys, ...] uint16 -> rows before the video, kept video rows, rows after it."""
    src = _u16(src)
    keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
    n_keys = src.shape[0]
    row = int(np.prod(src.shape[1:], dtype=np.int64))
    n_out = n_keys - n_video + keep_idx.shape[0]
    dst = np.zeros((n_out,) + src.shape[1:], dtype=np.uint16)
    rc = lib().oracle_gather_kv(_p(src), _p(dst), n_keys, video_start, n_video,
                                _p(keep_idx), keep_idx.shape[0], row)
    if rc:
        raise ValueError(f"oracle_gather_kv rc={rc}")
    return dst


def accept_greedy(target_logits, draft_tokens) -> Tuple[int, np.ndarray]:
    t = np.ascontiguousarray(target_logits, dtype=np.float32)
    x = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    gamma, vocab = t.shape[0] - 1, t.shape[1]
    n = C.c_int32(0)
    out = np.zeros(gamma + 1, dtype=np.int32)
    rc = lib().oracle_accept_greedy(_p(t), _p(x), gamma, vocab, C.byref(n), _p(out))
    if rc:
        raise ValueError(f"oracle_accept_greedy rc={rc}")
    return int(n.value), out


def accept_sample(target_logits, draft_logits, draft_tokens, uniforms, temperature: float = 1.0
                  ) -> Tuple[int, np.ndarray, np.ndarray]:
    t = np.ascontiguousarray(target_logits, dtype=np.float32)
    gamma, vocab = t.shape[0] - 1, t.shape[1]
    dl = np.ascontiguousarray(draft_logits, dtype=np.float32).reshape(gamma, vocab)
    x = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    n = C.c_int32(0)
    out = np.zeros(gamma + 1, dtype=np.int32)
    margins = np.zeros(gamma + 1, dtype=np.float64)
    rc = lib().oracle_accept_sample(_p(t), _p(dl), _p(x), _p(u), gamma, vocab,
                                    C.c_double(temperature), C.byref(n), _p(out), _p(margins))
    if rc:
        raise ValueError(f"oracle_accept_sample rc={rc}")
    return int(n.value), out, margins


def final_token_interval(target_logits, draft_logits, n: int, token: int, temperature: float = 1.0
                         ) -> Tuple[float, float]:
    """Normalised CDF interval [lo, hi) of `token` in the final draw after n accepted drafts."""
    t = np.ascontiguousarray(target_logits, dtype=np.float32)
    gamma, vocab = t.shape[0] - 1, t.shape[1]
    dl = np.ascontiguousarray(draft_logits, dtype=np.float32).reshape(gamma, vocab)
    lo, hi = C.c_double(0), C.c_double(0)
    rc = lib().oracle_final_token_interval(_p(t), _p(dl), n, gamma, vocab, C.c_double(temperature),
                                           token, C.byref(lo), C.byref(hi))
    if rc:
        raise ValueError(f"oracle_final_token_interval rc={rc}")
    return lo.value, hi.value


def tree_attn(q, k, v, mask, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Block of tree nodes: node t sees the context and the block nodes whose bit is set in mask[t]."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    q_len, hq, d = q.shape
    kv_len, hkv, _ = k.shape
    out = np.zeros((q_len, hq, d), dtype=np.float64)
    lse = np.zeros((q_len, hq), dtype=np.float64)
    rc = lib().oracle_tree_attn(_p(q), _p(k), _p(v), _p(mask), q_len, kv_len, hq, hkv, d,
                                C.c_double(scale), _p(out), _p(lse))
    if rc:
        raise ValueError(f"oracle_tree_attn rc={rc}")
    return out, lse


def accept_tree_greedy(target_logits, node_tokens, parent) -> Tuple[int, np.ndarray, np.ndarray]:
    t = np.ascontiguousarray(target_logits, dtype=np.float32)
    n_nodes, vocab = t.shape
    x = np.ascontiguousarray(node_tokens, dtype=np.int32)
    par = np.ascontiguousarray(parent, dtype=np.int32)
    n = C.c_int32(0)
    nodes = np.zeros(n_nodes, dtype=np.int32)
    out = np.zeros(n_nodes, dtype=np.int32)
    rc = lib().oracle_accept_tree_greedy(_p(t), _p(x), _p(par), n_nodes, vocab, C.byref(n), _p(nodes), _p(out))
    if rc:
        raise ValueError(f"oracle_accept_tree_greedy rc={rc}")
    return int(n.value), nodes, out


BASELINE_MODES = {"window-front": 0, "window-middle": 1, "window-end": 2, "uniform": 3,
                  "frame-drop": 4, "lattice": 5, "random": 6, "uniform-per-frame": 7}


def splitmix64(seed: int, j: int) -> int:
    fn = lib().oracle_splitmix64
    fn.restype = C.c_uint64
    fn.argtypes = [C.c_uint64, C.c_uint64]
    return int(fn(seed, j))


def baseline_keep(mode: str, n_video: int, keep_budget: int, *, n_frames: int = 0, grid_h: int = 0,
                  grid_w: int = 0, stride_h: int = 1, stride_w: int = 1, seed: int = 0) -> np.ndarray:
    """Attention-agnostic retention set of the named ablation pruner -> ascending int32 indices."""
    buf = np.zeros(max(n_video, 1), dtype=np.int32)
    fn = lib().oracle_baseline_keep
    fn.argtypes = [C.c_int] * 8 + [C.c_uint64, C.c_void_p]
    n = fn(BASELINE_MODES[mode], n_video, n_frames, grid_h, grid_w, keep_budget, stride_h, stride_w,
           seed, _p(buf))
    if n < 0:
        raise ValueError(f"oracle_baseline_keep rc={n}")
    return buf[:n].copy()
