// specvlm_gather_kv: build the draft's pruned KV cache (end of Sec. 3.2: the
// draft keeps V_R u V_U plus the language prompt; Self-SD setting: same
// parameters, pruned KV cache).  A pure row copy, bound by HBM bandwidth: a
// thread moves 16-byte chunks, a wave covers 1 KiB of contiguous source and
// destination, one launch covers K and V of every layer.  When a row has a
// power-of-two number of chunks (the usual head counts) the row and chunk of a
// thread are a shift and a mask instead of 64-bit divisions.
#include "common.h"

namespace specvlm {

struct GatherParams {
    const __bf16* src[2];
    __bf16* dst[2];
    int64_t src_layer, src_tok, src_head, dst_layer, dst_tok, dst_head;
    const int32_t* keep_idx;
    const int32_t* cu_keys;       // batch: prefix offsets of the requests' source rows, video tokens and
    const int32_t* cu_video;      //        kept tokens (device); all null for a single request
    const int32_t* cu_keep;
    int32_t* status;              // optional: set to SPECVLM_EINVAL when a request or an index is out of range
    int batch;
    int n_dst_rows, video_start, n_video, n_keep, n_kv_heads;
    int chunks_per_head;          // head_dim / 8
    int chunks_per_row;           // n_kv_heads * chunks_per_head
    int64_t chunks_per_layer;     // n_dst_rows * chunks_per_row
    int row_shift;                // log2(chunks_per_row) when that is a power of two, else -1
};

// Source row of destination row `row` (both counted over the whole batch), or -1 when the row has
// no valid source: a kept index outside its request's video span, or a request whose sizes do not
// fit together.  Such rows are zero-filled and reported through the status word.
__device__ __forceinline__ int gather_src_row(const GatherParams& p, int row)
{
    int src0 = 0, n_keys = p.n_dst_rows - p.n_keep + p.n_video, n_video = p.n_video, n_keep = p.n_keep, keep0 = 0;
    if (p.cu_keys) {
        // request b owns destination rows [off(b), off(b+1)), off(b) = cu_keys[b] - cu_video[b] + cu_keep[b]
        int lo = 0, hi = p.batch;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (row >= p.cu_keys[mid] - p.cu_video[mid] + p.cu_keep[mid]) lo = mid; else hi = mid;
        }
        src0 = p.cu_keys[lo]; keep0 = p.cu_keep[lo];
        n_keys = p.cu_keys[lo + 1] - src0;
        n_video = p.cu_video[lo + 1] - p.cu_video[lo];
        n_keep = p.cu_keep[lo + 1] - keep0;
        row -= src0 - p.cu_video[lo] + keep0;
        if (n_video < 0 || n_keep < 0 || n_keep > n_video || p.video_start + n_video > n_keys) {
            if (p.status) *p.status = SPECVLM_EINVAL;
            return -1;
        }
    }
    if (row < p.video_start) return src0 + row;
    if (row < p.video_start + n_keep) {
        const int j = p.keep_idx[keep0 + row - p.video_start];
        if (j < 0 || j >= n_video) {
            if (p.status) *p.status = SPECVLM_EINVAL;
            return -1;
        }
        return src0 + p.video_start + j;
    }
    return src0 + row - n_keep + n_video;
}

__global__ void gather_status_clear_kernel(int32_t* status) { *status = SPECVLM_OK; }

__global__ __launch_bounds__(256)
void gather_kernel(const GatherParams p)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.chunks_per_layer) return;
    const int layer = blockIdx.y, which = blockIdx.z;
    const int row = (int)(idx / p.chunks_per_row);
    const int ch = (int)(idx % p.chunks_per_row);
    const int head = ch / p.chunks_per_head, e = (ch % p.chunks_per_head) * 8;
    const int src_row = gather_src_row(p, row);
    const __bf16* s = p.src[which] + layer * p.src_layer + (int64_t)(src_row < 0 ? 0 : src_row) * p.src_tok +
                      (int64_t)head * p.src_head + e;
    __bf16* d = p.dst[which] + layer * p.dst_layer + (int64_t)row * p.dst_tok +
                (int64_t)head * p.dst_head + e;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (src_row >= 0) x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s));
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(d));
}

// chunks_per_row = 2^row_shift: a workgroup covers kGatherRowsPerThread * R consecutive rows
// (R = 256 >> row_shift), thread (r, ch) the chunk ch of rows r, r + R, ... of that group.  One row
// per thread: many small workgroups in flight beat more loads per thread here (8.6 us against
// 10.7 us with four rows per thread for 2 x 18.5 MB).
constexpr int kGatherRowsPerThread = 1;
__global__ __launch_bounds__(256)
void gather_pow2_kernel(const GatherParams p)
{
    const int layer = blockIdx.y, which = blockIdx.z;
    const int rows_per_pass = 256 >> p.row_shift;
    const int ch = threadIdx.x & ((1 << p.row_shift) - 1);
    const int head = ch / p.chunks_per_head, e = (ch % p.chunks_per_head) * 8;
    const int row0 = blockIdx.x * (kGatherRowsPerThread * rows_per_pass) + (threadIdx.x >> p.row_shift);
    const __bf16* sb = p.src[which] + layer * p.src_layer + (int64_t)head * p.src_head + e;
    __bf16* db = p.dst[which] + layer * p.dst_layer + (int64_t)head * p.dst_head + e;
    int src_row[kGatherRowsPerThread];
    bool live[kGatherRowsPerThread];
#pragma unroll
    for (int j = 0; j < kGatherRowsPerThread; ++j) {
        const int row = row0 + j * rows_per_pass;
        live[j] = row < p.n_dst_rows;
        src_row[j] = live[j] ? gather_src_row(p, row) : -1;
    }
    u32x4 x[kGatherRowsPerThread];
#pragma unroll
    for (int j = 0; j < kGatherRowsPerThread; ++j) {
        x[j] = u32x4{0u, 0u, 0u, 0u};                  // a row without a valid source is zero-filled
        if (src_row[j] >= 0)
            x[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(sb + (int64_t)src_row[j] * p.src_tok));
    }
#pragma unroll
    for (int j = 0; j < kGatherRowsPerThread; ++j)
        if (live[j])
            __builtin_nontemporal_store(x[j], reinterpret_cast<u32x4*>(db + (int64_t)(row0 + j * rows_per_pass) * p.dst_tok));
}

}  // namespace specvlm

using namespace specvlm;

extern "C" int specvlm_gather_kv(
    const void* k_src, const void* v_src,
    int64_t src_layer_stride, int64_t src_tok_stride, int64_t src_head_stride,
    void* k_dst, void* v_dst,
    int64_t dst_layer_stride, int64_t dst_tok_stride, int64_t dst_head_stride,
    int n_layers, int n_keys, int video_start, int n_video,
    const int32_t* keep_idx, int n_keep,
    const int32_t* cu_keys, const int32_t* cu_video, const int32_t* cu_keep, int batch,
    int32_t* status, int n_kv_heads, int head_dim, void* stream)
{
    if (n_layers < 0 || n_keys < 0 || video_start < 0 || n_video < 0 || n_keep < 0 || n_kv_heads <= 0 || batch < 0)
        return SPECVLM_EINVAL;
    const bool have_cu = cu_keys || cu_video || cu_keep;
    if (have_cu && !(cu_keys && cu_video && cu_keep)) return SPECVLM_EINVAL;
    if (!have_cu && batch > 1) return SPECVLM_EINVAL;
    if (batch == 0) return SPECVLM_OK;
    if ((int64_t)video_start + n_video > n_keys || n_keep > n_video) return SPECVLM_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SPECVLM_EUNSUPPORTED;
    if ((v_src == nullptr) != (v_dst == nullptr)) return SPECVLM_EINVAL;
    const int n_dst = n_keys - n_video + n_keep;
    const bool empty = n_layers == 0 || n_dst == 0;
    if (!empty && (!k_src || !k_dst || (n_keep > 0 && !keep_idx))) return SPECVLM_EINVAL;
    if ((src_layer_stride | src_tok_stride | src_head_stride | dst_layer_stride | dst_tok_stride |
         dst_head_stride) & 7)
        return SPECVLM_EUNSUPPORTED;
    if (((uintptr_t)k_src | (uintptr_t)k_dst | (uintptr_t)v_src | (uintptr_t)v_dst) & 15)
        return SPECVLM_EUNSUPPORTED;
    if (n_layers > 65535) return SPECVLM_EUNSUPPORTED;
    if (status) hipLaunchKernelGGL(gather_status_clear_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, status);
    if (empty) return launch_status();

    GatherParams p;
    p.src[0] = (const __bf16*)k_src; p.src[1] = (const __bf16*)v_src;
    p.dst[0] = (__bf16*)k_dst; p.dst[1] = (__bf16*)v_dst;
    p.src_layer = src_layer_stride; p.src_tok = src_tok_stride; p.src_head = src_head_stride;
    p.dst_layer = dst_layer_stride; p.dst_tok = dst_tok_stride; p.dst_head = dst_head_stride;
    p.keep_idx = keep_idx;
    p.cu_keys = cu_keys; p.cu_video = cu_video; p.cu_keep = cu_keep; p.status = status; p.batch = batch;
    p.n_dst_rows = n_dst; p.video_start = video_start; p.n_video = n_video; p.n_keep = n_keep;
    p.n_kv_heads = n_kv_heads;
    p.chunks_per_head = head_dim / 8;
    p.chunks_per_row = n_kv_heads * p.chunks_per_head;
    p.chunks_per_layer = (int64_t)n_dst * p.chunks_per_row;
    const int64_t blocks = (p.chunks_per_layer + 255) / 256;
    if (blocks > 0x7fffffff) return SPECVLM_EUNSUPPORTED;
    p.row_shift = -1;
    for (int sh = 0; sh <= 8; ++sh)
        if (p.chunks_per_row == (1 << sh)) p.row_shift = sh;
    if (p.row_shift >= 0) {
        const int rows_per_wg = kGatherRowsPerThread * (256 >> p.row_shift);
        dim3 grid((unsigned)((n_dst + rows_per_wg - 1) / rows_per_wg), (unsigned)n_layers, v_src ? 2u : 1u);
        hipLaunchKernelGGL(gather_pow2_kernel, grid, dim3(256), 0, (hipStream_t)stream, p);
    } else {
        dim3 grid((unsigned)blocks, (unsigned)n_layers, v_src ? 2u : 1u);
        hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, (hipStream_t)stream, p);
    }
    return launch_status();
}
