// specvlm_baseline_keep: retention sets of the attention-agnostic pruners the
// paper's ablations run against SpecVLM (Sec. 2.2: random pruning; Sec. 5.2:
// windows over the front, middle and end of the video; SD-Uniform, also restarted
// per frame or as a 2-D lattice; SD-Frame).
// Every mode except the random one is a closed form of the output position, so
// one thread writes one index.  The random mode draws one SplitMix64 output
// per token (counter-based: output j of the stream depends on (seed, j) only),
// turns its 30 high bits into a positive finite fp32 whose order is the
// integer's order, and lets the Stage-I radix select keep the B largest.
#include "common.h"

namespace specvlm {

struct BaselineParams {
    int mode;
    int n_video, n_frames, grid_h, grid_w, keep_budget, stride_h, stride_w;
    int count;
    int32_t* keep_idx;
};

__global__ __launch_bounds__(256)
void baseline_index_kernel(const BaselineParams p)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= p.count) return;
    const int64_t V = p.n_video, B = p.keep_budget;
    const int tpf = p.grid_h * p.grid_w;
    int64_t idx = 0;
    switch (p.mode) {
    case SPECVLM_BASELINE_WINDOW_FRONT:  idx = t; break;
    case SPECVLM_BASELINE_WINDOW_MIDDLE: idx = (V - B) / 2 + t; break;
    case SPECVLM_BASELINE_WINDOW_END:    idx = V - B + t; break;
    case SPECVLM_BASELINE_UNIFORM:       idx = ((int64_t)t * V) / B; break;
    case SPECVLM_BASELINE_FRAME_DROP: {
        const int64_t fk = B / tpf;                       // whole frames kept
        const int64_t slot = t / tpf, within = t % tpf;
        idx = ((slot * p.n_frames) / fk) * tpf + within;
        break;
    }
    case SPECVLM_BASELINE_LATTICE: {
        const int ch = (p.grid_h + p.stride_h - 1) / p.stride_h;
        const int cw = (p.grid_w + p.stride_w - 1) / p.stride_w;
        const int f = t / (ch * cw), rem = t % (ch * cw);
        idx = (int64_t)f * tpf + (int64_t)(rem / cw) * p.stride_h * p.grid_w + (rem % cw) * p.stride_w;
        break;
    }
    case SPECVLM_BASELINE_UNIFORM_PER_FRAME: {
        // output position t belongs to the frame f with floor(f*B/F) <= t < floor((f+1)*B/F)
        const int64_t F = p.n_frames;
        const int64_t f = ((int64_t)(t + 1) * F - 1) / B;
        const int64_t lo = (f * B) / F, hi = ((f + 1) * B) / F;
        idx = f * tpf + ((t - lo) * tpf) / (hi - lo);
        break;
    }
    default: break;
    }
    p.keep_idx[t] = (int32_t)idx;
}

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// draws[j] = the 30 high bits of output j, as the fp32 with that bit pattern (below 2.0, never
// NaN or infinite: float order == integer order); sizes[0..1] = the budget, for the select kernel.
__global__ __launch_bounds__(256)
void baseline_draw_kernel(uint64_t seed, int n_video, int keep_budget, float* draws, int32_t* sizes)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j == 0) { sizes[0] = keep_budget; sizes[1] = keep_budget; }
    if (j >= n_video) return;
    draws[j] = __uint_as_float((uint32_t)(splitmix64_at(seed, (uint64_t)j) >> 34));
}

}  // namespace specvlm

using namespace specvlm;

extern "C" int specvlm_baseline_count(int mode, int n_video, int n_frames, int grid_h, int grid_w,
                                      int keep_budget, int stride_h, int stride_w)
{
    if (n_video < 0 || keep_budget < 0 || keep_budget > n_video) return SPECVLM_EINVAL;
    switch (mode) {
    case SPECVLM_BASELINE_WINDOW_FRONT:
    case SPECVLM_BASELINE_WINDOW_MIDDLE:
    case SPECVLM_BASELINE_WINDOW_END:
    case SPECVLM_BASELINE_UNIFORM:
        return keep_budget;
    case SPECVLM_BASELINE_RANDOM:
        return n_video > 65536 ? SPECVLM_EUNSUPPORTED : keep_budget;
    case SPECVLM_BASELINE_FRAME_DROP:
    case SPECVLM_BASELINE_LATTICE:
    case SPECVLM_BASELINE_UNIFORM_PER_FRAME: {
        if (n_frames < 0 || grid_h <= 0 || grid_w <= 0) return SPECVLM_EINVAL;
        const int64_t tpf = (int64_t)grid_h * grid_w;
        if (tpf * n_frames != n_video) return SPECVLM_EINVAL;
        if (mode == SPECVLM_BASELINE_UNIFORM_PER_FRAME) return keep_budget;
        if (mode == SPECVLM_BASELINE_FRAME_DROP) return (int)((keep_budget / tpf) * tpf);
        if (stride_h <= 0 || stride_w <= 0) return SPECVLM_EINVAL;
        return n_frames * ((grid_h + stride_h - 1) / stride_h) * ((grid_w + stride_w - 1) / stride_w);
    }
    default:
        return SPECVLM_EINVAL;
    }
}

extern "C" size_t specvlm_baseline_workspace_bytes(int mode, int n_video)
{
    if (mode != SPECVLM_BASELINE_RANDOM || n_video <= 0) return 0;
    return align256((size_t)n_video * sizeof(float)) + 256;
}

extern "C" int specvlm_baseline_keep(int mode, int n_video, int n_frames, int grid_h, int grid_w,
                                     int keep_budget, int stride_h, int stride_w, uint64_t seed,
                                     int32_t* keep_idx, void* workspace, size_t workspace_bytes,
                                     void* stream)
{
    const int count = specvlm_baseline_count(mode, n_video, n_frames, grid_h, grid_w, keep_budget,
                                             stride_h, stride_w);
    if (count < 0) return count;
    if (count == 0) return SPECVLM_OK;
    if (!keep_idx) return SPECVLM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (mode == SPECVLM_BASELINE_RANDOM) {
        const size_t need = specvlm_baseline_workspace_bytes(mode, n_video);
        if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SPECVLM_EWORKSPACE;
        float* draws = (float*)workspace;
        int32_t* sizes = (int32_t*)((char*)workspace + align256((size_t)n_video * sizeof(float)));
        hipLaunchKernelGGL(baseline_draw_kernel, dim3((n_video + 255) / 256), dim3(256), 0, st,
                           seed, n_video, keep_budget, draws, sizes);
        int rc = launch_status();
        if (rc != SPECVLM_OK) return rc;
        // Stage I alone with k = B: the B largest draws, equal draws by lower index
        return specvlm_select(draws, nullptr, sizes, sizes + 1, nullptr, 1, n_video, keep_budget,
                              keep_idx, nullptr, nullptr, nullptr, 0, stream);
    }
    BaselineParams p;
    p.mode = mode; p.n_video = n_video; p.n_frames = n_frames; p.grid_h = grid_h; p.grid_w = grid_w;
    p.keep_budget = keep_budget; p.stride_h = stride_h; p.stride_w = stride_w;
    p.count = count; p.keep_idx = keep_idx;
    hipLaunchKernelGGL(baseline_index_kernel, dim3((count + 255) / 256), dim3(256), 0, st, p);
    return launch_status();
}
