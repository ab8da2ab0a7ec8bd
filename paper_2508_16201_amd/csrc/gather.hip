// specvlm_gather_kv: build the draft's pruned KV cache (end of Sec. 3.2: the
// draft keeps V_R u V_U plus the language prompt; Self-SD setting: same
// parameters, pruned KV cache).  A pure row copy, bound by HBM bandwidth: each
// thread moves one 16-byte chunk, a wave covers 1 KiB of contiguous source and
// destination, one launch covers K and V of every layer.
#include "common.h"

namespace specvlm {

struct GatherParams {
    const __bf16* src[2];
    __bf16* dst[2];
    int64_t src_layer, src_tok, src_head, dst_layer, dst_tok, dst_head;
    const int32_t* keep_idx;
    int n_dst_rows, video_start, n_video, n_keep, n_kv_heads;
    int chunks_per_head;          // head_dim / 8
    int chunks_per_row;           // n_kv_heads * chunks_per_head
    int64_t chunks_per_layer;     // n_dst_rows * chunks_per_row
};

__global__ __launch_bounds__(256)
void gather_kernel(const GatherParams p)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.chunks_per_layer) return;
    const int layer = blockIdx.y, which = blockIdx.z;
    const int row = (int)(idx / p.chunks_per_row);
    const int ch = (int)(idx % p.chunks_per_row);
    const int head = ch / p.chunks_per_head, e = (ch % p.chunks_per_head) * 8;
    int src_row;
    if (row < p.video_start) src_row = row;
    else if (row < p.video_start + p.n_keep)     // indices are clamped into the video span
        src_row = p.video_start + min(max(p.keep_idx[row - p.video_start], 0), p.n_video - 1);
    else src_row = row - p.n_keep + p.n_video;
    const __bf16* s = p.src[which] + layer * p.src_layer + (int64_t)src_row * p.src_tok +
                      (int64_t)head * p.src_head + e;
    __bf16* d = p.dst[which] + layer * p.dst_layer + (int64_t)row * p.dst_tok +
                (int64_t)head * p.dst_head + e;
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s));
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(d));
}

}  // namespace specvlm

using namespace specvlm;

extern "C" int specvlm_gather_kv(
    const void* k_src, const void* v_src,
    int64_t src_layer_stride, int64_t src_tok_stride, int64_t src_head_stride,
    void* k_dst, void* v_dst,
    int64_t dst_layer_stride, int64_t dst_tok_stride, int64_t dst_head_stride,
    int n_layers, int n_keys, int video_start, int n_video,
    const int32_t* keep_idx, int n_keep, int n_kv_heads, int head_dim, void* stream)
{
    if (n_layers < 0 || n_keys < 0 || video_start < 0 || n_video < 0 || n_keep < 0 || n_kv_heads <= 0)
        return SPECVLM_EINVAL;
    if ((int64_t)video_start + n_video > n_keys || n_keep > n_video) return SPECVLM_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SPECVLM_EUNSUPPORTED;
    if ((v_src == nullptr) != (v_dst == nullptr)) return SPECVLM_EINVAL;
    const int n_dst = n_keys - n_video + n_keep;
    if (n_layers == 0 || n_dst == 0) return SPECVLM_OK;
    if (!k_src || !k_dst || (n_keep > 0 && !keep_idx)) return SPECVLM_EINVAL;
    if ((src_layer_stride | src_tok_stride | src_head_stride | dst_layer_stride | dst_tok_stride |
         dst_head_stride) & 7)
        return SPECVLM_EUNSUPPORTED;
    if (((uintptr_t)k_src | (uintptr_t)k_dst | (uintptr_t)v_src | (uintptr_t)v_dst) & 15)
        return SPECVLM_EUNSUPPORTED;
    if (n_layers > 65535) return SPECVLM_EUNSUPPORTED;

    GatherParams p;
    p.src[0] = (const __bf16*)k_src; p.src[1] = (const __bf16*)v_src;
    p.dst[0] = (__bf16*)k_dst; p.dst[1] = (__bf16*)v_dst;
    p.src_layer = src_layer_stride; p.src_tok = src_tok_stride; p.src_head = src_head_stride;
    p.dst_layer = dst_layer_stride; p.dst_tok = dst_tok_stride; p.dst_head = dst_head_stride;
    p.keep_idx = keep_idx;
    p.n_dst_rows = n_dst; p.video_start = video_start; p.n_video = n_video; p.n_keep = n_keep;
    p.n_kv_heads = n_kv_heads;
    p.chunks_per_head = head_dim / 8;
    p.chunks_per_row = n_kv_heads * p.chunks_per_head;
    p.chunks_per_layer = (int64_t)n_dst * p.chunks_per_row;
    const int64_t blocks = (p.chunks_per_layer + 255) / 256;
    if (blocks > 0x7fffffff) return SPECVLM_EUNSUPPORTED;
    dim3 grid((unsigned)blocks, (unsigned)n_layers, v_src ? 2u : 1u);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, (hipStream_t)stream, p);
    return launch_status();
}
