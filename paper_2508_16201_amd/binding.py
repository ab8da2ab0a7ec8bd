"""ctypes binding of ``libspecvlm.so``: argument marshalling only.

Every function has the name of the C entry point it calls (``include/specvlm.h``)
and takes torch tensors that live on the GPU; torch provides device memory and
the current stream, nothing else.  There is no CPU fallback: if the HIP
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPECVLM_LIB names another build of the same library (the host-sanitized one the CPU tests make)
LIB_PATH = os.environ.get("SPECVLM_LIB") or os.path.join(_HERE, "libspecvlm.so")
_lib = None

EXPORTS = (
    "specvlm_status_string", "specvlm_version",
    "specvlm_score_workspace_bytes", "specvlm_score",
    "specvlm_score_layers_workspace_bytes", "specvlm_score_layers",
    "specvlm_select_workspace_bytes", "specvlm_select",
    "specvlm_top_p_count_workspace_bytes", "specvlm_top_p_count",
    "specvlm_gather_kv",
    "specvlm_decode_attn_workspace_bytes", "specvlm_decode_attn",
    "specvlm_decode_attn_static_scratch_bytes", "specvlm_decode_attn_static",
    "specvlm_accept_workspace_bytes", "specvlm_accept",
    "specvlm_tree_attn", "specvlm_accept_tree_workspace_bytes", "specvlm_accept_tree",
    "specvlm_baseline_count", "specvlm_baseline_workspace_bytes", "specvlm_baseline_keep",
    "specvlm_probe_read",
)


class SpecVLMError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {status_string(status)} ({status})")


def lib() -> C.CDLL:
    """Load the HIP library (built by ``paper_2508_16201_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2508_16201_amd.build` "
                "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        l.specvlm_status_string.restype = C.c_char_p
        l.specvlm_status_string.argtypes = [C.c_int]
        l.specvlm_version.restype = C.c_int
        for name in EXPORTS:
            if name.endswith("_workspace_bytes") or name.endswith("_scratch_bytes"):
                getattr(l, name).restype = C.c_size_t
        i64, i32, f32, vp, sz = C.c_int64, C.c_int, C.c_float, C.c_void_p, C.c_size_t
        l.specvlm_score_workspace_bytes.argtypes = [i32] * 8
        l.specvlm_score.argtypes = [vp, i64, i64, vp, i64, i64, vp, vp, vp, i32,
                                    i32, i32, i32, i32, i32, i32, i32, i32, f32,
                                    i32, vp, f32, vp, vp, sz, vp]
        l.specvlm_score_layers_workspace_bytes.argtypes = [i32] * 9
        l.specvlm_score_layers.argtypes = [vp, i64, i64, i64, vp, i64, i64, i64, i32, vp, vp, vp, i32,
                                           i32, i32, i32, i32, i32, i32, i32, i32, f32,
                                           i32, vp, i64, f32, vp, vp, sz, vp]
        l.specvlm_select_workspace_bytes.argtypes = [i32, i32]
        l.specvlm_select.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        l.specvlm_top_p_count_workspace_bytes.argtypes = [i32, i32]
        l.specvlm_top_p_count.argtypes = [vp, vp, i32, i32, f32, vp, vp, vp, sz, vp]
        l.specvlm_gather_kv.argtypes = [vp, vp, i64, i64, i64, vp, vp, i64, i64, i64,
                                        i32, i32, i32, i32, vp, i32, vp, vp, vp, i32, vp, i32, i32, vp]
        l.specvlm_decode_attn_workspace_bytes.argtypes = [i32] * 7
        l.specvlm_decode_attn.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32, i32, i32,
                                          i32, i32, i32, f32, vp, vp, i32, vp, sz, vp]
        l.specvlm_decode_attn_static_scratch_bytes.argtypes = []
        l.specvlm_decode_attn_static.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32, i32, i32,
                                                 i32, i32, i32, f32, vp, vp, i32, vp]
        l.specvlm_tree_attn.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32, i32, i32,
                                        i32, i32, i32, f32, vp, vp, vp, i32, vp, sz, vp]
        l.specvlm_accept_tree_workspace_bytes.argtypes = [i32] * 3
        l.specvlm_accept_tree.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        l.specvlm_baseline_count.argtypes = [i32] * 8
        l.specvlm_baseline_count.restype = C.c_int
        l.specvlm_baseline_workspace_bytes.argtypes = [i32] * 2
        l.specvlm_baseline_keep.argtypes = [i32] * 8 + [C.c_uint64, vp, vp, sz, vp]
        l.specvlm_baseline_keep.restype = C.c_int
        l.specvlm_probe_read.argtypes = [vp, sz, vp, sz, vp, vp]
        l.specvlm_probe_read.restype = C.c_int
        l.specvlm_accept_workspace_bytes.argtypes = [i32] * 4
        l.specvlm_accept.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, sz, vp]
        for name in ("specvlm_score", "specvlm_select", "specvlm_top_p_count", "specvlm_gather_kv",
                     "specvlm_decode_attn", "specvlm_decode_attn_static", "specvlm_accept", "specvlm_tree_attn",
                     "specvlm_accept_tree"):
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().specvlm_status_string(int(status)).decode()


def version() -> int:
    return lib().specvlm_version()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensors must live on the GPU")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn: str, rc: int):
    if rc != 0:
        raise SpecVLMError(fn, rc)


def new_workspace(nbytes: int, device=None) -> torch.Tensor:
    """A 256-byte aligned device buffer (torch's caching allocator aligns to 512)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device or "cuda")


def _ws(workspace: Optional[torch.Tensor], need: int, like: torch.Tensor) -> torch.Tensor:
    if workspace is None:
        workspace = new_workspace(need, like.device)
    return workspace


def _thd(t: torch.Tensor) -> Tuple[int, int]:
    """(token stride, head stride) in elements of a [tokens, heads, d] view."""
    if t.dim() != 3 or t.stride(2) != 1:
        raise ValueError("expected a [tokens, heads, d] view with contiguous d")
    return t.stride(0), t.stride(1)


# --------------------------------------------------------------------------- score
def score_workspace_bytes(n_text, n_keys, n_video, n_q_heads, n_kv_heads, head_dim,
                          have_row_lse=False, batch=1) -> int:
    return lib().specvlm_score_workspace_bytes(batch, n_text, n_keys, n_video, n_q_heads, n_kv_heads,
                                               head_dim, int(have_row_lse))


def score_layers_workspace_bytes(n_layers, n_text, n_keys, n_video, n_q_heads, n_kv_heads, head_dim,
                                 have_row_lse=False, batch=1) -> int:
    return lib().specvlm_score_layers_workspace_bytes(n_layers, batch, n_text, n_keys, n_video, n_q_heads,
                                                      n_kv_heads, head_dim, int(have_row_lse))


def _dev_i32(a, device):
    """Device int32 prefix offsets; a host sequence is uploaded (and its maxima returned)."""
    if isinstance(a, torch.Tensor):
        return a, None
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    return torch.from_numpy(arr).to(device), arr


def _batch_sizes(device, cu_text, cu_keys, cu_video, n_text, n_keys, n_video, max_n_text, max_n_keys,
                 max_n_video, total_video):
    """(batch, device offset arrays, maxima, total video tokens) of a score call; one request without offsets."""
    if cu_text is None:
        return 1, (None, None, None), n_text, n_keys, n_video, n_video
    dev = [_dev_i32(a, device) for a in (cu_text, cu_keys, cu_video)]
    ptrs = tuple(x[0] for x in dev)
    batch = ptrs[0].numel() - 1
    hosts = [x[1] for x in dev]
    if all(h is not None for h in hosts):
        n_text = int(np.diff(hosts[0]).max()) if batch else 0
        n_keys = int(np.diff(hosts[1]).max()) if batch else 0
        n_video = int(np.diff(hosts[2]).max()) if batch else 0
        total_video = int(hosts[2][-1])
    else:
        if None in (max_n_text, max_n_keys, max_n_video, total_video):
            raise ValueError("device cu arrays need max_n_text, max_n_keys, max_n_video and total_video")
        n_text, n_keys, n_video = max_n_text, max_n_keys, max_n_video
    return batch, ptrs, n_text, n_keys, n_video, total_video


def score_layers(q_text: torch.Tensor, k_cache: torch.Tensor, video_start: int, n_video: int,
                 text_pos0: int, softmax_scale: float, *, norm_mode: int = 0,
                 row_lse: Optional[torch.Tensor] = None, beta: float = 0.0,
                 scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 cu_text=None, cu_keys=None, cu_video=None, max_n_text: Optional[int] = None,
                 max_n_keys: Optional[int] = None, max_n_video: Optional[int] = None,
                 total_video: Optional[int] = None) -> torch.Tensor:
    """q_text [layers,L,H_q,d] bf16, k_cache [layers,n_keys,H_kv,d] bf16 (any layer / token / head strides with
    contiguous d), row_lse [layers,L,H_q] fp32 or None -> scores fp32 [n_video] summed over the layers.
    A batch is given as for score(): requests concatenated along the token axis of every layer."""
    n_layers, n_text, hq, d = q_text.shape
    _, n_keys, hkv, _ = k_cache.shape
    if k_cache.shape[0] != n_layers:
        raise ValueError("q_text and k_cache must have the same number of layers")
    if q_text.stride(3) != 1 or k_cache.stride(3) != 1:
        raise ValueError("the head dimension must be contiguous")
    if row_lse is not None and (row_lse.shape != (n_layers, n_text, hq) or not row_lse[0].is_contiguous()):
        raise ValueError("row_lse must be [layers, n_text, H_q] with contiguous layers")
    batch, ptrs, n_text, n_keys, n_video, total_video = _batch_sizes(
        q_text.device, cu_text, cu_keys, cu_video, n_text, n_keys, n_video, max_n_text, max_n_keys, max_n_video,
        total_video)
    if scores is None:
        scores = torch.empty(total_video, dtype=torch.float32, device=q_text.device)
        if beta != 0.0:
            raise ValueError("beta != 0 needs an existing scores tensor")
    need = score_layers_workspace_bytes(n_layers, n_text, n_keys, n_video, hq, hkv, d, row_lse is not None,
                                        batch=max(batch, 1))
    workspace = _ws(workspace, need, q_text)
    rc = lib().specvlm_score_layers(_ptr(q_text), q_text.stride(0), q_text.stride(1), q_text.stride(2),
                                    _ptr(k_cache), k_cache.stride(0), k_cache.stride(1), k_cache.stride(2), n_layers,
                                    _ptr(ptrs[0]), _ptr(ptrs[1]), _ptr(ptrs[2]), batch, n_text, n_keys, video_start,
                                    n_video, text_pos0, hq, hkv, d,
                                    float(softmax_scale), norm_mode, _ptr(row_lse),
                                    0 if row_lse is None else row_lse.stride(0), float(beta), _ptr(scores),
                                    _ptr(workspace), workspace.numel(), _stream())
    _check("specvlm_score_layers", rc)
    return scores


def score(q_text: torch.Tensor, k_cache: torch.Tensor, video_start: int, n_video: int,
          text_pos0: int, softmax_scale: float, *, norm_mode: int = 0,
          row_lse: Optional[torch.Tensor] = None, beta: float = 0.0,
          scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
          cu_text=None, cu_keys=None, cu_video=None, max_n_text: Optional[int] = None,
          max_n_keys: Optional[int] = None, max_n_video: Optional[int] = None,
          total_video: Optional[int] = None) -> torch.Tensor:
    """q_text [L,H_q,d] bf16, k_cache [n_keys,H_kv,d] bf16 -> scores fp32 [n_video].

    A batch: requests concatenated along the token axis, cu_text / cu_keys / cu_video = int32 prefix
    offsets [batch+1] on the device (host sequences are uploaded); n_video is then ignored and
    text_pos0 = -1 places every request's text queries on its last keys.  With device tensors the
    maxima over the batch and the total number of video tokens must be given."""
    n_text, hq, d = q_text.shape
    n_keys, hkv, _ = k_cache.shape
    batch, ptrs, n_text, n_keys, n_video, total_video = _batch_sizes(
        q_text.device, cu_text, cu_keys, cu_video, n_text, n_keys, n_video, max_n_text, max_n_keys, max_n_video,
        total_video)
    if scores is None:
        scores = torch.empty(total_video, dtype=torch.float32, device=q_text.device)
        if beta != 0.0:
            raise ValueError("beta != 0 needs an existing scores tensor")
    need = score_workspace_bytes(n_text, n_keys, n_video, hq, hkv, d, row_lse is not None, batch=max(batch, 1))
    workspace = _ws(workspace, need, q_text)
    qs, ks = _thd(q_text), _thd(k_cache)
    rc = lib().specvlm_score(_ptr(q_text), qs[0], qs[1], _ptr(k_cache), ks[0], ks[1],
                             _ptr(ptrs[0]), _ptr(ptrs[1]), _ptr(ptrs[2]), batch, n_text, n_keys, video_start,
                             n_video, text_pos0, hq, hkv, d, float(softmax_scale), norm_mode, _ptr(row_lse),
                             float(beta), _ptr(scores), _ptr(workspace), workspace.numel(), _stream())
    _check("specvlm_score", rc)
    return scores


# -------------------------------------------------------------------------- select
def select(scores: torch.Tensor, k_top: torch.Tensor, keep_budget: torch.Tensor, total_keep: int,
           *, cu_video: Optional[torch.Tensor] = None, cu_keep: Optional[torch.Tensor] = None,
           max_n_video: Optional[int] = None, want_flags: bool = True, want_status: bool = False,
           keep_idx: Optional[torch.Tensor] = None):
    """scores fp32 [sum V_b]; k_top/keep_budget device int32 [batch] -> keep_idx int32 [total_keep]."""
    batch = k_top.numel()
    if max_n_video is None:
        if cu_video is not None:
            raise ValueError("max_n_video is required with cu_video")
        max_n_video = scores.numel()
    dev = scores.device
    if keep_idx is None:
        keep_idx = torch.empty(total_keep, dtype=torch.int32, device=dev)
    flags = torch.empty(total_keep, dtype=torch.uint8, device=dev) if want_flags else None
    status = torch.empty(batch, dtype=torch.int32, device=dev) if want_status else None
    rc = lib().specvlm_select(_ptr(scores), _ptr(cu_video), _ptr(k_top), _ptr(keep_budget),
                              _ptr(cu_keep), batch, max_n_video, total_keep, _ptr(keep_idx),
                              _ptr(flags), _ptr(status), None, 0, _stream())
    _check("specvlm_select", rc)
    out = (keep_idx, flags)
    return out + (status,) if want_status else out


def top_p_count(scores: torch.Tensor, lam: float, *, cu_video: Optional[torch.Tensor] = None,
                max_n_video: Optional[int] = None, max_count: Optional[torch.Tensor] = None,
                count: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores fp32 [sum V_b] -> count int32 [batch]: Eq. 6's retention size per request."""
    batch = 1 if cu_video is None else cu_video.numel() - 1
    if max_n_video is None:
        if cu_video is not None:
            raise ValueError("max_n_video is required with cu_video")
        max_n_video = scores.numel()
    if count is None:
        count = torch.empty(batch, dtype=torch.int32, device=scores.device)
    rc = lib().specvlm_top_p_count(_ptr(scores), _ptr(cu_video), batch, max_n_video, float(lam),
                                   _ptr(max_count), _ptr(count), None, 0, _stream())
    _check("specvlm_top_p_count", rc)
    return count


# ----------------------------------------------------------------------- gather_kv
def gather_kv(k_src: torch.Tensor, v_src: Optional[torch.Tensor], video_start: int, n_video: int,
              keep_idx: torch.Tensor, k_dst: Optional[torch.Tensor] = None,
              v_dst: Optional[torch.Tensor] = None, *, cu_keys: Optional[torch.Tensor] = None,
              cu_video: Optional[torch.Tensor] = None, cu_keep: Optional[torch.Tensor] = None,
              want_status: bool = False):
    """k_src/v_src bf16 [layers, n_keys, H_kv, d] (any layer/token/head strides, d contiguous).

    A batch: requests concatenated along the token axis, cu_keys / cu_video / cu_keep device int32
    [batch+1]; n_video is then the total over the batch."""
    if k_src.dim() != 4 or k_src.stride(3) != 1:
        raise ValueError("expected [layers, tokens, heads, d] with contiguous d")
    n_layers, n_keys, hkv, d = k_src.shape
    n_keep = keep_idx.numel()
    n_dst = n_keys - n_video + n_keep
    batch = 1 if cu_keys is None else cu_keys.numel() - 1
    if k_dst is None:
        k_dst = torch.empty((n_layers, n_dst, hkv, d), dtype=k_src.dtype, device=k_src.device)
    if v_src is not None and v_dst is None:
        v_dst = torch.empty_like(k_dst)
    if v_src is not None and v_src.stride() != k_src.stride():
        raise ValueError("K and V must share strides")
    if v_dst is not None and v_dst.stride() != k_dst.stride():
        raise ValueError("K and V destinations must share strides")
    status = torch.empty(1, dtype=torch.int32, device=k_src.device) if want_status else None
    rc = lib().specvlm_gather_kv(_ptr(k_src), _ptr(v_src), k_src.stride(0), k_src.stride(1),
                                 k_src.stride(2), _ptr(k_dst), _ptr(v_dst), k_dst.stride(0),
                                 k_dst.stride(1), k_dst.stride(2), n_layers, n_keys, video_start,
                                 n_video, _ptr(keep_idx), n_keep, _ptr(cu_keys), _ptr(cu_video),
                                 _ptr(cu_keep), batch, _ptr(status), hkv, d, _stream())
    _check("specvlm_gather_kv", rc)
    return (k_dst, v_dst, status) if want_status else (k_dst, v_dst)


# --------------------------------------------------------------------- decode_attn
def decode_attn_workspace_bytes(batch, q_len, kv_len, n_q_heads, n_kv_heads, head_dim,
                                num_splits=0) -> int:
    return lib().specvlm_decode_attn_workspace_bytes(batch, q_len, kv_len, n_q_heads, n_kv_heads,
                                                     head_dim, num_splits)


def decode_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, softmax_scale: float, *,
                cu_q: Optional[torch.Tensor] = None, cu_kv: Optional[torch.Tensor] = None,
                max_q_len: Optional[int] = None, max_kv_len: Optional[int] = None,
                out: Optional[torch.Tensor] = None, want_lse: bool = False, num_splits: int = 0,
                workspace: Optional[torch.Tensor] = None, ancestor_mask: Optional[torch.Tensor] = None):
    """q [sum q_len,H_q,d], k/v [sum kv_len,H_kv,d] bf16 views -> out like q (and lse fp32)."""
    tq, hq, d = q.shape
    tk, hkv, _ = k.shape
    if cu_q is None:
        batch, q_len, kv_len = 1, tq, tk
    else:
        batch = cu_q.numel() - 1
        if max_q_len is None or max_kv_len is None:
            raise ValueError("max_q_len and max_kv_len are required with cu_q/cu_kv")
        q_len, kv_len = max_q_len, max_kv_len
    if out is None:
        out = torch.empty_like(q)
    if out.stride() != q.stride():
        raise ValueError("out must share q's strides")
    if v.stride() != k.stride():
        raise ValueError("K and V must share strides")
    lse = torch.empty((tq, hq), dtype=torch.float32, device=q.device) if want_lse else None
    need = decode_attn_workspace_bytes(batch, q_len, kv_len, hq, hkv, d, num_splits)
    workspace = _ws(workspace, need, q)
    qs, ks = _thd(q), _thd(k)
    if ancestor_mask is None:
        rc = lib().specvlm_decode_attn(_ptr(q), qs[0], qs[1], _ptr(k), _ptr(v), ks[0], ks[1],
                                       _ptr(cu_q), _ptr(cu_kv), batch, q_len, kv_len, hq, hkv, d,
                                       float(softmax_scale), _ptr(out), _ptr(lse), num_splits,
                                       _ptr(workspace), workspace.numel(), _stream())
        _check("specvlm_decode_attn", rc)
    else:
        rc = lib().specvlm_tree_attn(_ptr(q), qs[0], qs[1], _ptr(k), _ptr(v), ks[0], ks[1],
                                     _ptr(cu_q), _ptr(cu_kv), batch, q_len, kv_len, hq, hkv, d,
                                     float(softmax_scale), _ptr(ancestor_mask), _ptr(out), _ptr(lse),
                                     num_splits, _ptr(workspace), workspace.numel(), _stream())
        _check("specvlm_tree_attn", rc)
    return (out, lse) if want_lse else out


def decode_attn_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, softmax_scale: float, *,
                       out: torch.Tensor, lse: Optional[torch.Tensor] = None,
                       cu_q: Optional[torch.Tensor] = None, cu_kv: Optional[torch.Tensor] = None,
                       max_q_len: Optional[int] = None, max_kv_len: Optional[int] = None,
                       num_splits: int = 0) -> torch.Tensor:
    """decode_attn through the entry point that takes no workspace; the caller supplies every output
    (this wrapper allocates nothing either)."""
    tq, hq, d = q.shape
    tk, hkv, _ = k.shape
    if cu_q is None:
        batch, q_len, kv_len = 1, tq, tk
    else:
        batch = cu_q.numel() - 1
        if max_q_len is None or max_kv_len is None:
            raise ValueError("max_q_len and max_kv_len are required with cu_q/cu_kv")
        q_len, kv_len = max_q_len, max_kv_len
    if out.stride() != q.stride() or v.stride() != k.stride():
        raise ValueError("out must share q's strides, V must share K's")
    qs, ks = _thd(q), _thd(k)
    rc = lib().specvlm_decode_attn_static(_ptr(q), qs[0], qs[1], _ptr(k), _ptr(v), ks[0], ks[1],
                                          _ptr(cu_q), _ptr(cu_kv), batch, q_len, kv_len, hq, hkv, d,
                                          float(softmax_scale), _ptr(out), _ptr(lse), num_splits, _stream())
    _check("specvlm_decode_attn_static", rc)
    return out


def tree_attn(q, k, v, softmax_scale, ancestor_mask: torch.Tensor, **kw):
    """decode_attn for a block of draft-tree nodes; ancestor_mask int64/uint64 [sum q_len]."""
    return decode_attn(q, k, v, softmax_scale, ancestor_mask=ancestor_mask, **kw)


# -------------------------------------------------------------------------- accept
def accept_workspace_bytes(batch, gamma, vocab, sampling) -> int:
    return lib().specvlm_accept_workspace_bytes(batch, gamma, vocab, int(sampling))


def accept(target_logits: torch.Tensor, draft_tokens: torch.Tensor, *,
           draft_logits: Optional[torch.Tensor] = None, uniforms: Optional[torch.Tensor] = None,
           temperature: float = 1.0, workspace: Optional[torch.Tensor] = None,
           n_accepted: Optional[torch.Tensor] = None, out_tokens: Optional[torch.Tensor] = None):
    """target_logits fp32 [batch, gamma+1, vocab] -> (n_accepted int32 [batch], out_tokens int32 [batch, gamma+1])."""
    batch, g1, vocab = target_logits.shape
    gamma = g1 - 1
    dev = target_logits.device
    n_acc = n_accepted if n_accepted is not None else torch.empty(batch, dtype=torch.int32, device=dev)
    out = out_tokens if out_tokens is not None else \
        torch.empty((batch, gamma + 1), dtype=torch.int32, device=dev)
    sampling = uniforms is not None
    need = accept_workspace_bytes(batch, gamma, vocab, sampling)
    workspace = _ws(workspace, need, target_logits)
    for t in (target_logits, draft_logits, draft_tokens, uniforms):
        if t is not None and not t.is_contiguous():
            raise ValueError("accept inputs must be contiguous")
    rc = lib().specvlm_accept(_ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens),
                              _ptr(uniforms), batch, gamma, vocab, float(temperature),
                              _ptr(n_acc), _ptr(out), _ptr(workspace), workspace.numel(), _stream())
    _check("specvlm_accept", rc)
    return n_acc, out


def accept_tree(target_logits: torch.Tensor, node_tokens: torch.Tensor, parent: torch.Tensor, *,
                workspace: Optional[torch.Tensor] = None):
    """target_logits fp32 [batch, n_nodes, vocab], node_tokens int32 [batch, n_nodes], parent int32 [n_nodes]
    -> (n_accepted [batch], accepted_nodes [batch, n_nodes], out_tokens [batch, n_nodes])."""
    batch, n_nodes, vocab = target_logits.shape
    dev = target_logits.device
    n_acc = torch.empty(batch, dtype=torch.int32, device=dev)
    nodes = torch.empty((batch, n_nodes), dtype=torch.int32, device=dev)
    out = torch.empty((batch, n_nodes), dtype=torch.int32, device=dev)
    need = lib().specvlm_accept_tree_workspace_bytes(batch, n_nodes, vocab)
    workspace = _ws(workspace, need, target_logits)
    for t in (target_logits, node_tokens, parent):
        if not t.is_contiguous():
            raise ValueError("accept_tree inputs must be contiguous")
    rc = lib().specvlm_accept_tree(_ptr(target_logits), _ptr(node_tokens), _ptr(parent), batch, n_nodes,
                                   vocab, _ptr(n_acc), _ptr(nodes), _ptr(out), _ptr(workspace),
                                   workspace.numel(), _stream())
    _check("specvlm_accept_tree", rc)
    return n_acc, nodes, out


# ------------------------------------------------------------------- baseline pruners
BASELINE_MODES = {"window-front": 0, "window-middle": 1, "window-end": 2, "uniform": 3,
                  "frame-drop": 4, "lattice": 5, "random": 6, "uniform-per-frame": 7}


def baseline_keep(mode: str, n_video: int, keep_budget: int, *, n_frames: int = 0, grid_h: int = 0,
                  grid_w: int = 0, stride_h: int = 1, stride_w: int = 1, seed: int = 0,
                  device=None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Retention set of the named attention-agnostic pruner -> ascending int32 indices on the device."""
    m = BASELINE_MODES[mode]
    count = lib().specvlm_baseline_count(m, n_video, n_frames, grid_h, grid_w, keep_budget, stride_h, stride_w)
    if count < 0:
        raise SpecVLMError("specvlm_baseline_count", count)
    keep_idx = torch.empty(count, dtype=torch.int32, device=device or "cuda")
    need = lib().specvlm_baseline_workspace_bytes(m, n_video)
    if need:
        workspace = _ws(workspace, need, keep_idx)
    rc = lib().specvlm_baseline_keep(m, n_video, n_frames, grid_h, grid_w, keep_budget, stride_h, stride_w,
                                     seed, _ptr(keep_idx), _ptr(workspace),
                                     workspace.numel() if workspace is not None else 0, _stream())
    _check("specvlm_baseline_keep", rc)
    return keep_idx


# ------------------------------------------------------------------------ diagnostics
def probe_read(a: torch.Tensor, b: Optional[torch.Tensor] = None) -> None:
    """One launch that merely reads the bytes of `a` (and `b`): the bare-read yardstick of the benchmark.
    Both must be dense in memory (any dimension order)."""
    def span(t):
        if t is None:
            return None, 0
        return C.c_void_p(t.data_ptr()), t.numel() * t.element_size()
    pa, na = span(a)
    pb, nb = span(b)
    _check("specvlm_probe_read", lib().specvlm_probe_read(pa, na, pb, nb, None, _stream()))
