// specvlm_score: language-to-video attention scores (Sec. 3.1, Eq. 4-5).
//
//   a_j = (1/(H_q L)) sum_h sum_i softmax_row(scale * Q_L K^T)[i, j],  j in video
//
// The attention matrix is never materialised.  Two MFMA sweeps over the same
// text x key contraction:
//   pass A  row statistics: for every (text query, q head) row the running
//           (max, sum exp) over the keys of the normalisation domain, split over
//           key ranges and merged -> log2-domain normaliser lse2[row]
//           (skipped when the caller supplies row_lse);
//   pass B  column sums: for every video key, sum over rows of
//           exp2(logit2 - lse2[row]), split over row ranges;
//   final   scores = beta*scores + mean over (h, i), summing the kv-head / split
//           partials in a fixed order (deterministic, no float atomics).
//
// Both passes are one kernel template.  A workgroup (4 waves) keeps 256
// "stationary" vectors (rows of Q in pass A, video keys in pass B) as MFMA
// B-operand fragments in registers, 64 per wave, and streams the other side
// through an LDS ring of 64-vector tiles filled by direct-to-LDS loads
// (XOR-swizzled 16-byte chunks).  In the accumulator layout the stationary
// vector is lane column r and the streamed vectors are rows 4c..4c+3, so each
// pass reduces over its streamed side inside a lane and needs no cross-lane
// traffic until the very end.
//
// Rows of one kv head are indexed sigma = gl * L_pad + i (q head gl of the
// group, text query i, L_pad = L rounded up to the tile size): a streamed tile
// of pass B therefore holds 64 consecutive queries of ONE q head and its
// addresses need no per-lane division.
//
// The exponentials dominate the arithmetic (one v_exp_f32 per logit, quarter
// rate); pass A keeps them to one per logit by rescaling its running sum only
// when a tile's maximum exceeds the reference by more than 2^8.
#include "common.h"

namespace specvlm {

#define SPECVLM_AS1 __attribute__((address_space(1)))
#define SPECVLM_AS3 __attribute__((address_space(3)))

constexpr int kScoreTile = 64;         // streamed vectors per LDS tile
constexpr int kScoreBlock = 256;       // stationary vectors per workgroup
constexpr int kScoreStages = 3;        // LDS ring depth
constexpr float kNegBig = -1.0e30f;    // finite stand-in for "no key seen yet"
constexpr float kLazyMargin = 8.f;     // log2 units of headroom before the running sum is rescaled

struct ScoreParams {
    const __bf16* q;
    const __bf16* k;
    int64_t q_tok, q_head, k_tok, k_head;
    int n_text, n_keys, video_start, n_video, text_pos0;
    int n_q_heads, n_kv_heads, group;
    float scale_log2;
    int l_pad;                     // n_text rounded up to the tile size
    int rows, rows_pad;            // rows = group * l_pad (per kv head), padded to 256
    int video_pad;                 // n_video padded to 256
    int key_lo, key_hi;            // normalisation domain [key_lo, key_hi)
    int a_splits, a_split_keys;
    int b_splits, b_split_rows;
    int b_needs_mask;
    float* part_ml;                // [H_kv][rows_pad][a_splits][2]
    float* lse2;                   // [H_kv][rows_pad]
    const float* row_lse;          // caller's natural-log normalisers [n_text][H_q], or null
    float* part_cols;              // [H_kv][b_splits][video_pad]
    float beta, inv_count;
    float* scores;
};

constexpr int score_vmcnt_imm(int n)
{
    return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8);
}

template <int D, int MODE>
__global__ __launch_bounds__(256)
void score_sweep_kernel(const ScoreParams p)
{
    constexpr int KK = D / 32;
    constexpr int CH = D / 8;                        // 16-byte chunks per vector
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = kScoreTile * ROW_BYTES;
    constexpr int VEC_PER_LOAD = kWave / CH;         // vectors one wave-wide load covers
    constexpr int LPW = kScoreTile / VEC_PER_LOAD / 4;   // loads per wave per tile (4 waves)
    constexpr int NS = kScoreStages;
    __shared__ __align__(16) unsigned char s_tile[NS][TILE_BYTES];
    __shared__ __align__(16) float s_lse[NS][kScoreTile];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, c = lane >> 4;
    // Workgroups go to the XCDs round-robin by linear id.  Decode the id so that
    // the stationary blocks of one (kv head, split) are neighbours on ONE XCD:
    // they stream the same tiles at the same time and share them in that L2.
    const int n_blocks = (MODE == 0 ? p.rows_pad : p.video_pad) / kScoreBlock;
    const int n_split = (MODE == 0 ? p.a_splits : p.b_splits);
    const int vid = xcd_logical_id(blockIdx.x, gridDim.x);
    if (vid >= n_blocks * n_split * p.n_kv_heads) return;
    const int blk = vid % n_blocks;
    const int split = (vid / n_blocks) % n_split;
    const int g = vid / (n_blocks * n_split);
    const int stat0 = blk * kScoreBlock + wave * 64;             // this wave's first stationary vector

    // streamed range of this workgroup (multiples of the tile size)
    int s_begin, s_end;
    if (MODE == 0) {
        s_begin = p.key_lo + split * p.a_split_keys;
        s_end = min(p.key_hi, s_begin + p.a_split_keys);
    } else {
        s_begin = split * p.b_split_rows;
        s_end = min(p.rows, s_begin + p.b_split_rows);
    }

    // ---- stationary fragments (B operand) ----
    bf16x8 sf[4][KK];
    int lim[4];                                 // pass A: last visible key of the lane's row
    int key_abs[4];                             // pass B: absolute key index of the lane's key
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) {
        const int item = stat0 + sb * 16 + r;
        const __bf16* src = nullptr;
        lim[sb] = -1; key_abs[sb] = 0x7fffffff;
        if (MODE == 0) {
            const int gl = item / p.l_pad, i = item % p.l_pad;
            if (item < p.rows && i < p.n_text) {
                src = p.q + (int64_t)i * p.q_tok + (int64_t)(g * p.group + gl) * p.q_head;
                lim[sb] = p.text_pos0 + i;
            }
        } else {
            if (item < p.n_video) {
                key_abs[sb] = p.video_start + item;
                src = p.k + (int64_t)key_abs[sb] * p.k_tok + (int64_t)g * p.k_head;
            }
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (src) raw = *reinterpret_cast<const u32x4*>(src + kk * 32 + c * 8);
            sf[sb][kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    float m_ref[4], l_run[4], col[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) { m_ref[sb] = kNegBig; l_run[sb] = 0.f; col[sb] = 0.f; }

    // ---- loader: direct-to-LDS, load j of a wave covers VEC_PER_LOAD vectors ----
    const int ld_vec = lane / CH, ld_chunk = lane % CH;
    auto issue_tile = [&](int tile, int stage) {
        const int first = s_begin + tile * kScoreTile;
        // pass B: the tile holds consecutive text queries of one q head
        int gl = 0, i0 = 0;
        if (MODE == 1) { gl = first / p.l_pad; i0 = first % p.l_pad; }
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int n = wave + 4 * j;                          // load index inside the tile
            const int it = n * VEC_PER_LOAD + ld_vec;            // vector inside the tile
            const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
            const int chunk = ld_chunk ^ swz;
            const __bf16* src;
            if (MODE == 0) {
                const int key = min(first + it, p.n_keys - 1);   // rows past the range are masked later
                src = p.k + (int64_t)key * p.k_tok + (int64_t)g * p.k_head;
            } else {
                const int i = min(i0 + it, p.n_text - 1);        // padded rows carry lse = +inf
                src = p.q + (int64_t)i * p.q_tok + (int64_t)(g * p.group + gl) * p.q_head;
            }
            __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)(src + chunk * 8),
                                             (SPECVLM_AS3 void*)(&s_tile[stage][n * 1024]), 16, 0, 0);
        }
        if (MODE == 1 && wave == 0) {
            // the tile's 64 row normalisers (+inf for padded rows), one dword per lane
            const float* src = p.lse2 + (int64_t)g * p.rows_pad + first + lane;
            __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)src,
                                             (SPECVLM_AS3 void*)(&s_lse[stage][0]), 4, 0, 0);
        }
    };

    auto compute = [&](int stage, int first) {
        bool mask = false;
        if (MODE == 0) {
            // earliest text query among the workgroup's rows sees keys <= text_pos0
            mask = (first + kScoreTile > s_end) || (first + kScoreTile - 1 > p.text_pos0);
        }
#pragma unroll 1
        for (int sub = 0; sub < 4; ++sub) {
            bf16x8 af[KK];
            const int it = sub * 16 + r;
            const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int x = kk * 4 + c;
                af[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                    &s_tile[stage][it * ROW_BYTES + ((x ^ swz) * 16)]));
            }
            floatx4 acc[4];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                acc[sb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) acc[sb] = mfma16(af[kk], sf[sb][kk], acc[sb]);
            }
            if (MODE == 0) {
                // (a zero scale is taken as a vanishing one, so that a masked logit, -inf, times the
                // scale stays -inf instead of becoming NaN; every other logit still scales to 0)
                const float sc_a = fmaxf(p.scale_log2, 1e-30f);
                float tmax[4];
#pragma unroll
                for (int sb = 0; sb < 4; ++sb) {
                    if (mask) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int key = first + sub * 16 + 4 * c + i;
                            if (key >= s_end || key > lim[sb]) acc[sb][i] = -INFINITY;
                        }
                    }
                    // the logits stay unscaled: the scale (>= 0) is applied to the maximum once and
                    // rides in the fused multiply-add that forms each exponent
                    tmax[sb] = fmaxf(fmaxf(acc[sb][0], acc[sb][1]), fmaxf(acc[sb][2], acc[sb][3])) * p.scale_log2;
                }
                // rescale only when some row's new maximum outgrows its reference
                bool grow = false;
#pragma unroll
                for (int sb = 0; sb < 4; ++sb) grow = grow || (tmax[sb] > m_ref[sb] + kLazyMargin);
                if (__any(grow)) {
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        const float m_new = fmaxf(m_ref[sb], tmax[sb]);
                        l_run[sb] *= fast_exp2(m_ref[sb] - m_new);
                        m_ref[sb] = m_new;
                    }
                }
#pragma unroll
                for (int sb = 0; sb < 4; ++sb) {
                    const float sc = sc_a, mr = m_ref[sb];
                    const float sum = (fast_exp2(fmaf(acc[sb][0], sc, -mr)) + fast_exp2(fmaf(acc[sb][1], sc, -mr))) +
                                      (fast_exp2(fmaf(acc[sb][2], sc, -mr)) + fast_exp2(fmaf(acc[sb][3], sc, -mr)));
                    l_run[sb] += sum;
                }
            } else {
                const floatx4 lse4 = *reinterpret_cast<const floatx4*>(&s_lse[stage][sub * 16 + 4 * c]);
                if (p.b_needs_mask) {
                    // text query i of this tile sees keys <= text_pos0 + i
                    const int lim0 = p.text_pos0 + (first % p.l_pad) + sub * 16 + 4 * c;
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        float sum = 0.f;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float pr = fast_exp2(acc[sb][i] * p.scale_log2 - lse4[i]);
                            sum += (key_abs[sb] > lim0 + i) ? 0.f : pr;
                        }
                        col[sb] += sum;
                    }
                } else {
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        const float sum = (fast_exp2(acc[sb][0] * p.scale_log2 - lse4[0]) +
                                           fast_exp2(acc[sb][1] * p.scale_log2 - lse4[1])) +
                                          (fast_exp2(acc[sb][2] * p.scale_log2 - lse4[2]) +
                                           fast_exp2(acc[sb][3] * p.scale_log2 - lse4[3]));
                        col[sb] += sum;
                    }
                }
            }
        }
    };

    // ---- ring: NS-1 tiles in flight while one is consumed; one barrier per tile ----
    const int n_tiles = (s_end - s_begin + kScoreTile - 1) / kScoreTile;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < n_tiles) issue_tile(s, s);
    for (int t = 0; t < n_tiles; ++t) {
        const int younger = min(NS - 2, n_tiles - 1 - t);
        // (wave 0 of pass B has one more load per tile: it waits slightly longer than needed)
        if (younger >= 1) __builtin_amdgcn_s_waitcnt(score_vmcnt_imm(LPW) & ~(15 << 8));
        else __builtin_amdgcn_s_waitcnt(score_vmcnt_imm(0) & ~(15 << 8));
        __asm__ volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __asm__ volatile("" ::: "memory");
        if (t + NS - 1 < n_tiles) issue_tile(t + NS - 1, (t + NS - 1) % NS);
        compute(t % NS, s_begin + t * kScoreTile);
    }

    // ---- reduce over the four lane groups that share a stationary vector ----
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) {
        const int item = stat0 + sb * 16 + r;
        if (MODE == 0) {
            float m = m_ref[sb], l = l_run[sb];
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                const float om = __shfl_xor(m, off), ol = __shfl_xor(l, off);
                const float mm = fmaxf(m, om);
                l = l * fast_exp2(m - mm) + ol * fast_exp2(om - mm);
                m = mm;
            }
            if (c == 0 && item < p.rows) {
                float* dst = p.part_ml + (((int64_t)g * p.rows_pad + item) * p.a_splits + split) * 2;
                dst[0] = m; dst[1] = l;
            }
        } else {
            float v = col[sb];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (c == 0 && item < p.n_video)
                p.part_cols[((int64_t)g * p.b_splits + split) * p.video_pad + item] = v;
        }
    }
}

// lse2[g][row] from the pass-A partials, or from the caller's natural-log values.
__global__ __launch_bounds__(256)
void score_lse_kernel(const ScoreParams p)
{
    const int row = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
    if (row >= p.rows_pad) return;
    float out = INFINITY;                       // padded / keyless rows contribute nothing
    const int gl = row / p.l_pad, i = row % p.l_pad;
    if (row < p.rows && i < p.n_text) {
        if (p.row_lse) {
            out = p.row_lse[(int64_t)i * p.n_q_heads + g * p.group + gl] * kLog2e;
            if (!(out > -INFINITY)) out = INFINITY;
        } else {
            const float* src = p.part_ml + ((int64_t)g * p.rows_pad + row) * p.a_splits * 2;
            float m = kNegBig;
            for (int s = 0; s < p.a_splits; ++s) m = fmaxf(m, src[2 * s]);
            float l = 0.f;
            for (int s = 0; s < p.a_splits; ++s) l += src[2 * s + 1] * fast_exp2(src[2 * s] - m);
            if (l > 0.f) out = m + fast_log2(l);
        }
    }
    p.lse2[(int64_t)g * p.rows_pad + row] = out;
}

__global__ __launch_bounds__(256)
void score_final_kernel(const ScoreParams p)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p.n_video) return;
    float a = 0.f;
    const int parts = p.n_kv_heads * p.b_splits;
    for (int s = 0; s < parts; ++s) a += p.part_cols[(int64_t)s * p.video_pad + j];
    a *= p.inv_count;
    p.scores[j] = (p.beta != 0.f ? p.beta * p.scores[j] : 0.f) + a;
}

struct ScorePlan {
    int l_pad, rows, rows_pad, video_pad, key_lo, key_hi, a_splits, a_split_keys, b_splits, b_split_rows;
    size_t off_ml, off_lse, off_cols, total;
};

static ScorePlan score_plan(int n_text, int n_keys, int video_start, int n_video, int n_q_heads,
                            int n_kv_heads, int norm_mode, int have_row_lse)
{
    ScorePlan s;
    const int group = n_q_heads / n_kv_heads;
    s.l_pad = round_up(n_text > 0 ? n_text : 1, kScoreTile);
    s.rows = group * s.l_pad;
    s.rows_pad = round_up(s.rows, kScoreBlock);
    s.video_pad = round_up(n_video > 0 ? n_video : 1, kScoreBlock);
    s.key_lo = norm_mode ? video_start : 0;
    s.key_hi = norm_mode ? video_start + n_video : n_keys;
    // Three workgroups fit a CU (48 KB of LDS ring, < 170 VGPRs).  A split count is
    // good when the workgroups fill whole rounds of those slots: minimise
    // rounds x tiles-per-workgroup, ties to the fewer splits (less partial traffic).
    const int slots = 3 * kNumCu;
    auto best_splits = [&](int blocks, int streamed, int max_splits, int* per_split) {
        int best = 1, best_per = round_up(streamed > 0 ? streamed : 1, kScoreTile);
        long best_cost = -1;
        for (int n = 1; n <= max_splits; ++n) {
            const int per = round_up((streamed + n - 1) / n > 0 ? (streamed + n - 1) / n : 1, kScoreTile);
            const int live = streamed > 0 ? (streamed + per - 1) / per : 1;
            if (live != n) continue;                             // same partition as a smaller n
            const long wgs = (long)blocks * live;
            const long rounds = (wgs + slots - 1) / slots;
            // +2 tiles: a workgroup's fixed cost (stationary fragments, ring fill); + live: fewer splits on ties
            const long cost = rounds * (per / kScoreTile + 2) * 64 + live;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = live; best_per = per; }
        }
        *per_split = best_per;
        return best;
    };
    const int dom = s.key_hi - s.key_lo;
    const int blocks_a = (s.rows_pad / kScoreBlock) * n_kv_heads;
    s.a_splits = best_splits(blocks_a, dom, 64, &s.a_split_keys);
    const int blocks_b = (s.video_pad / kScoreBlock) * n_kv_heads;
    s.b_splits = best_splits(blocks_b, s.rows, 16, &s.b_split_rows);
    size_t off = 0;
    s.off_ml = off;
    if (!have_row_lse) off += align256((size_t)n_kv_heads * s.rows_pad * s.a_splits * 2 * sizeof(float));
    s.off_lse = off;  off += align256((size_t)n_kv_heads * s.rows_pad * sizeof(float));
    s.off_cols = off; off += align256((size_t)n_kv_heads * s.b_splits * s.video_pad * sizeof(float));
    s.total = off;
    return s;
}

}  // namespace specvlm

using namespace specvlm;

extern "C" size_t specvlm_score_workspace_bytes(int batch, int n_text, int n_keys, int n_video,
                                                int n_q_heads, int n_kv_heads, int head_dim,
                                                int have_row_lse)
{
    (void)head_dim;
    if (batch != 1 || n_text < 0 || n_keys < 0 || n_video < 0 || n_video > n_keys ||
        n_kv_heads <= 0 || n_q_heads <= 0 || n_q_heads % n_kv_heads)
        return 0;
    // the split plan depends on the normalisation domain; size for the larger one
    const ScorePlan a = score_plan(n_text, n_keys, 0, n_video, n_q_heads, n_kv_heads, 0, have_row_lse);
    const ScorePlan b = score_plan(n_text, n_keys, 0, n_video, n_q_heads, n_kv_heads, 1, have_row_lse);
    return a.total > b.total ? a.total : b.total;
}

extern "C" int specvlm_score(
    const void* q_text,  int64_t q_tok_stride, int64_t q_head_stride,
    const void* k_cache, int64_t k_tok_stride, int64_t k_head_stride,
    const int32_t* cu_text, const int32_t* cu_keys, const int32_t* cu_video, int batch,
    int n_text, int n_keys, int video_start, int n_video, int text_pos0,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    int norm_mode, const float* row_lse, float beta, float* scores,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch < 0 || n_text < 0 || n_keys < 0 || video_start < 0 || n_video < 0 || text_pos0 < 0)
        return SPECVLM_EINVAL;
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads) return SPECVLM_EINVAL;
    if ((int64_t)video_start + n_video > n_keys) return SPECVLM_EINVAL;
    if (norm_mode != 0 && norm_mode != 1) return SPECVLM_EINVAL;
    if (!(softmax_scale >= 0.f) || !(softmax_scale < INFINITY)) return SPECVLM_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SPECVLM_EUNSUPPORTED;
    if (batch == 0 || n_video == 0) return SPECVLM_OK;
    if (cu_text || cu_keys || cu_video || batch != 1) return SPECVLM_EUNSUPPORTED;   // one request per call
    if (!scores) return SPECVLM_EINVAL;
    if (n_text > 0 && (!q_text || !k_cache)) return SPECVLM_EINVAL;
    if ((q_tok_stride | q_head_stride | k_tok_stride | k_head_stride) & 7) return SPECVLM_EUNSUPPORTED;
    if (((uintptr_t)q_text | (uintptr_t)k_cache) & 15) return SPECVLM_EUNSUPPORTED;

    const ScorePlan plan = score_plan(n_text, n_keys, video_start, n_video, n_q_heads, n_kv_heads,
                                      norm_mode, row_lse != nullptr);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < plan.total) return SPECVLM_EWORKSPACE;

    ScoreParams p;
    p.q = (const __bf16*)q_text; p.k = (const __bf16*)k_cache;
    p.q_tok = q_tok_stride; p.q_head = q_head_stride; p.k_tok = k_tok_stride; p.k_head = k_head_stride;
    p.n_text = n_text; p.n_keys = n_keys; p.video_start = video_start; p.n_video = n_video;
    p.text_pos0 = text_pos0;
    p.n_q_heads = n_q_heads; p.n_kv_heads = n_kv_heads; p.group = n_q_heads / n_kv_heads;
    p.scale_log2 = softmax_scale * kLog2e;
    p.l_pad = plan.l_pad;
    p.rows = plan.rows; p.rows_pad = plan.rows_pad; p.video_pad = plan.video_pad;
    p.key_lo = plan.key_lo; p.key_hi = plan.key_hi;
    p.a_splits = plan.a_splits; p.a_split_keys = plan.a_split_keys;
    p.b_splits = plan.b_splits; p.b_split_rows = plan.b_split_rows;
    p.b_needs_mask = (video_start + n_video - 1 > text_pos0) ? 1 : 0;
    p.part_ml = (float*)((char*)workspace + plan.off_ml);
    p.lse2 = (float*)((char*)workspace + plan.off_lse);
    p.row_lse = row_lse;
    p.part_cols = (float*)((char*)workspace + plan.off_cols);
    p.beta = beta;
    p.inv_count = (n_text > 0) ? 1.f / ((float)n_q_heads * (float)n_text) : 0.f;
    p.scores = scores;
    hipStream_t s = (hipStream_t)stream;

    if (n_text > 0) {
        if (!row_lse && p.key_hi > p.key_lo) {
            dim3 grid(round_up((plan.rows_pad / kScoreBlock) * n_kv_heads * plan.a_splits, kNumXcd));
            if (head_dim == 128) hipLaunchKernelGGL((score_sweep_kernel<128, 0>), grid, dim3(256), 0, s, p);
            else                 hipLaunchKernelGGL((score_sweep_kernel<64, 0>), grid, dim3(256), 0, s, p);
        }
        hipLaunchKernelGGL(score_lse_kernel, dim3(plan.rows_pad / 256, n_kv_heads), dim3(256), 0, s, p);
        dim3 grid(round_up((plan.video_pad / kScoreBlock) * n_kv_heads * plan.b_splits, kNumXcd));
        if (head_dim == 128) hipLaunchKernelGGL((score_sweep_kernel<128, 1>), grid, dim3(256), 0, s, p);
        else                 hipLaunchKernelGGL((score_sweep_kernel<64, 1>), grid, dim3(256), 0, s, p);
    } else {
        p.b_splits = 0;          // no language queries: the mean is empty, only beta applies
    }
    hipLaunchKernelGGL(score_final_kernel, dim3((n_video + 255) / 256), dim3(256), 0, s, p);
    return launch_status();
}
