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
// Per logit the VALU issues one fma, one v_exp_f32 (half rate) and one add, as
// much issue time as the logit's share of the MFMAs: the two streams are
// interleaved instruction by instruction inside a wave.  Pass A keeps to one
// exponential per logit: away from the causal mask it does not track maxima at
// all, and where it does it rescales its running sum only when a tile's maximum
// exceeds the reference by more than 2^8.
#include "common.h"

namespace specvlm {

#define SPECVLM_AS1 __attribute__((address_space(1)))
#define SPECVLM_AS3 __attribute__((address_space(3)))

constexpr int kScoreTile = 64;         // streamed vectors per LDS tile
constexpr int kScoreBlock = 256;       // stationary vectors per workgroup
constexpr int kScoreStages = 3;        // LDS ring depth
constexpr float kNegBig = -1.0e30f;    // finite stand-in for "no key seen yet"
constexpr int kMaxSplitsA = 64;        // key-range splits of pass A, at most
constexpr int kMaxSplitsB = 16;        // row-range splits of pass B, at most
constexpr float kLazyMargin = 8.f;     // log2 units of headroom before the running sum is rescaled
constexpr float kSumRedo = 0x1p100f;   // a running sum at or above this (or NaN) is recomputed with maxima tracked

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
    // a batch: device prefix offsets of the requests (null: one request, the scalars above are its sizes;
    // else the scalars are the maxima over the batch and the sizes of a request come from here)
    const int32_t* cu_text;
    const int32_t* cu_keys;
    const int32_t* cu_video;
    int batch, norm_mode;
    int64_t ws_ml, ws_lse, ws_cols;    // floats per (layer, request) in part_ml / lse2 / part_cols
    // several layers in one call: layer l reads q + l*q_layer, k + l*k_layer, row_lse + l*lse_layer and owns
    // the workspace slices l*batch .. l*batch + batch - 1; the final kernel sums the layers
    int n_layers;
    int64_t q_layer, k_layer, lse_layer;
};

// The view of (layer, request) number idx = layer * batch + b of the launch parameters: pointers moved
// to its layer and rows, sizes and positions its own.  The plan (padding, split sizes) stays that of
// the maxima, so a workgroup whose share lies beyond the request's real size finds an empty range.
// Returns false for a request whose sizes do not fit the maxima or each other: every kernel skips it.
__device__ __forceinline__ bool score_select_request(ScoreParams& p, int idx)
{
    const int layer = idx / p.batch, b = idx - layer * p.batch;
    p.part_ml += (int64_t)idx * p.ws_ml;
    p.lse2 += (int64_t)idx * p.ws_lse;
    p.part_cols += (int64_t)idx * p.ws_cols;
    p.q += layer * p.q_layer;
    p.k += layer * p.k_layer;
    if (p.row_lse) p.row_lse += layer * p.lse_layer;
    if (!p.cu_text) return true;
    const int t0 = p.cu_text[b], k0 = p.cu_keys[b], v0 = p.cu_video[b];
    const int nt = p.cu_text[b + 1] - t0, nk = p.cu_keys[b + 1] - k0, nv = p.cu_video[b + 1] - v0;
    if (nt < 0 || nk < 0 || nv < 0 || nt > p.n_text || nk > p.n_keys || nv > p.n_video ||
        p.video_start + nv > nk)
        return false;
    const int pos0 = p.text_pos0 >= 0 ? p.text_pos0 : nk - nt;      // -1: the text queries are the last keys
    if (pos0 < 0) return false;
    p.q += (int64_t)t0 * p.q_tok;
    p.k += (int64_t)k0 * p.k_tok;
    if (p.row_lse) p.row_lse += (int64_t)t0 * p.n_q_heads;
    p.scores += v0;
    p.n_text = nt; p.n_keys = nk; p.n_video = nv; p.text_pos0 = pos0;
    p.key_lo = p.norm_mode ? p.video_start : 0;
    p.key_hi = p.norm_mode ? p.video_start + nv : nk;
    p.b_needs_mask = (p.video_start + nv - 1 > pos0) ? 1 : 0;
    p.inv_count = nt > 0 ? 1.f / ((float)p.n_q_heads * (float)nt) : 0.f;
    return true;
}

constexpr int score_vmcnt_imm(int n)
{
    return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8);
}

// ---- pieces of one sub-block (16 streamed vectors x the wave's 64 stationary ones) ----
// A fragments of sub-block `sub` of the tile at `tile` (lane (r, c) reads streamed vector sub*16 + r)
template <int D>
__device__ __forceinline__ void score_load_a(const unsigned char* tile, int sub, int r, int c, bf16x8 (&af)[D / 32])
{
    const int it = sub * 16 + r;
    const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        const int x = kk * 4 + c;
        af[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(tile + it * (D * 2) + ((x ^ swz) * 16)));
    }
}

template <int KK>
__device__ __forceinline__ void score_mfma(const bf16x8 (&af)[KK], const bf16x8 (&sf)[4][KK], floatx4 (&acc)[4])
{
    // the four accumulators take turns, so that no MFMA waits for the one issued just before it
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
        for (int sb = 0; sb < 4; ++sb)
            acc[sb] = mfma16(af[kk], sf[sb][kk], kk == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[sb]);
    }
}

// pass A, first half: mask (key0 = the lane's first key of the sub-block), maxima per row, and the
// rare rescale of the running sums when some row's maximum outgrows its reference
__device__ __forceinline__ void score_rows_max(floatx4 (&acc)[4], bool mask, int key0, int s_end, const int (&lim)[4],
                                               float scale_log2, float (&m_ref)[4], float (&l_run)[4])
{
    float tmax[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) {
        if (mask) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (key0 + i >= s_end || key0 + i > lim[sb]) acc[sb][i] = -INFINITY;
        }
        // the logits stay unscaled: the scale (>= 0) is applied to the maximum once and rides in
        // the fused multiply-add that forms each exponent
        tmax[sb] = fmaxf(fmaxf(acc[sb][0], acc[sb][1]), fmaxf(acc[sb][2], acc[sb][3])) * scale_log2;
    }
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
}

// (register budget: three waves per SIMD, i.e. at most 168 VGPRs, which head size 128 needs all of)
template <int D, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void score_sweep_kernel(const ScoreParams p_launch)
{
    ScoreParams p = p_launch;
    constexpr int KK = D / 32;
    constexpr int CH = D / 8;                        // 16-byte chunks per vector
    constexpr int ROW_BYTES = D * 2;
    constexpr int TILE_BYTES = kScoreTile * ROW_BYTES;
    constexpr int VEC_PER_LOAD = kWave / CH;         // vectors one wave-wide load covers
    constexpr int LPW = kScoreTile / VEC_PER_LOAD / 4;   // loads per wave per tile (4 waves)
    constexpr int NS = kScoreStages;
    // One LDS object for everything the direct-to-LDS loads fill (the compiler orders reads of an
    // object after ALL loads in flight into it when it sees several such objects): NS tiles, then
    // per stage and wave a private copy of the tile's 64 row normalisers.
    constexpr int LSE_BYTES = kScoreTile * 4;
    __shared__ __align__(16) unsigned char s_mem[NS * TILE_BYTES + NS * 4 * LSE_BYTES];
    unsigned char* const s_tile = s_mem;
    unsigned char* const s_lse = s_mem + NS * TILE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, c = lane >> 4;
    // Workgroups go to the XCDs round-robin by linear id.  Decode the id so that
    // the stationary blocks of one (kv head, split) are neighbours on ONE XCD:
    // they stream the same tiles at the same time and share them in that L2.
    const int n_blocks = (MODE == 0 ? p.rows_pad : p.video_pad) / kScoreBlock;
    const int n_split = (MODE == 0 ? p.a_splits : p.b_splits);
    const int vid = xcd_logical_id(blockIdx.x, gridDim.x);
    if (vid >= n_blocks * n_split * p.n_kv_heads * p.batch * p.n_layers) return;
    const int blk = vid % n_blocks;
    const int split = (vid / n_blocks) % n_split;
    const int g = (vid / (n_blocks * n_split)) % p.n_kv_heads;
    if (!score_select_request(p, vid / (n_blocks * n_split * p.n_kv_heads))) return;
    const int stat0 = blk * kScoreBlock + wave * 64;             // this wave's first stationary vector

    // streamed range of this workgroup (multiples of the tile size)
    int s_begin, s_end;
    if (MODE == 0) {
        s_begin = min(p.key_hi, p.key_lo + split * p.a_split_keys);
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
    // The per-lane part of a load's address is the same for every tile: byte offset of the lane's
    // vector and chunk from the tile's first vector.  A tile then costs one scalar base address;
    // only a tile that runs past the last vector takes the per-lane clamped path.
    const int ld_vec = lane / CH, ld_chunk = lane % CH;
    const int64_t s_tok = (MODE == 0) ? p.k_tok : p.q_tok;       // streamed side: token stride (elements)
    uint32_t voff[LPW];
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int it = (wave + 4 * j) * VEC_PER_LOAD + ld_vec;   // vector inside the tile
        const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
        voff[j] = (uint32_t)it * (uint32_t)(s_tok * 2) + (uint32_t)((ld_chunk ^ swz) * 16);
    }
    // Tiles are requested in order; the position of the next one is carried along (pass B: text
    // query nx_idx0 of q head nx_gl) instead of being divided out of the tile index every time.
    const int n_tiles = (s_end - s_begin + kScoreTile - 1) / kScoreTile;
    int nx_tile = 0, nx_idx0 = s_begin, nx_gl = 0;
    if (MODE == 1) { nx_gl = s_begin / p.l_pad; nx_idx0 = s_begin % p.l_pad; }
    auto issue_next = [&](int stage) {
        // pass A streams keys of kv head g; pass B streams consecutive text queries of ONE q head
        const int idx0 = nx_idx0;
        const int limit = (MODE == 0) ? p.n_keys : p.n_text;
        const int64_t head_off = (MODE == 0) ? (int64_t)g * p.k_head : (int64_t)(g * p.group + nx_gl) * p.q_head;
        const __bf16* base = (MODE == 0) ? p.k : p.q;
        const int first = (MODE == 0) ? idx0 : nx_gl * p.l_pad + idx0;
        if (nx_tile + 1 < n_tiles) {          // past the end the last tile is requested again
            ++nx_tile;
            nx_idx0 += kScoreTile;
            if (MODE == 1 && nx_idx0 >= p.l_pad) { nx_idx0 = 0; ++nx_gl; }
        }
        if (idx0 + kScoreTile <= limit) {
            const char* tile_base = reinterpret_cast<const char*>(base + (int64_t)idx0 * s_tok + head_off);
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                // (the offset is made opaque here so that it stays one 32-bit register beside a scalar
                // base: seen through, it is widened to a 64-bit pair outside the loop)
                uint32_t off = voff[j];
                asm volatile("" : "+v"(off));
                __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)(tile_base + off),
                    (SPECVLM_AS3 void*)(s_tile + stage * TILE_BYTES + (wave + 4 * j) * 1024), 16, 0, 0);
            }
        } else {
            // vectors past the end are masked later (pass A) or carry lse = +inf (pass B): re-read the last one
            // (rare path: its lane constants are recomputed here instead of living in registers)
            int lv = ld_vec, lc = ld_chunk;
            asm volatile("" : "+v"(lv), "+v"(lc));
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                const int n = wave + 4 * j;
                const int it = n * VEC_PER_LOAD + lv;
                const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
                const int idx = min(idx0 + it, limit - 1);
                const __bf16* src = base + (int64_t)idx * s_tok + head_off + (lc ^ swz) * 8;
                __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)src,
                    (SPECVLM_AS3 void*)(s_tile + stage * TILE_BYTES + n * 1024), 16, 0, 0);
            }
        }
        if (MODE == 1) {
            // the tile's 64 row normalisers (+inf for padded rows), one dword per lane; every wave
            // fetches its own copy, so all waves have the same number of loads in flight per tile
            const float* src = p.lse2 + (int64_t)g * p.rows_pad + first + lane;
            __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)src,
                                             (SPECVLM_AS3 void*)(s_lse + (stage * 4 + wave) * LSE_BYTES), 4, 0, 0);
        }
    };

    // ---- one tile: 4 sub-blocks of 16 streamed vectors against the wave's 64 stationary ones ----
    // Software pipeline inside the wave: while the VALU turns the logits of sub-block s into
    // exponentials, the matrix unit already forms the logits of sub-block s+1 (independent MFMA and
    // VALU instructions of one wave overlap).  The order is written out piece by piece -- one MFMA,
    // one logit's fma / exp / add -- and pinned with scheduling barriers: left alone, the scheduler
    // moves every chain of MFMAs next to its consumer again.  Even sub-blocks accumulate in acc0, odd
    // ones in acc1.  There is ONE set of A fragments: fragment kk of sub-block s+2 is read from LDS
    // right after the last MFMA of sub-block s+1 that uses fragment kk, most of a sub-block before
    // its own first use.  (A second set, read a whole sub-block earlier, cost 16 registers and with
    // them the third wave per SIMD at head size 128.)
    // (a zero scale is taken as a vanishing one, so that a masked logit, -inf, times the scale stays
    // -inf instead of becoming NaN; every other logit still scales to 0)
    const float sc_a = fmaxf(p.scale_log2, 1e-30f);
    auto step = [&](floatx4 (&acc_cur)[4], floatx4 (&acc_nxt)[4], bf16x8 (&af)[KK],
                    const unsigned char* tile, const unsigned char* lse_w, const int sub, const int first,
                    const int lim0, const bool mask, const bool track, const bool has_next, const bool has_load)
        __attribute__((always_inline)) {
        floatx4 lse4 = {0.f, 0.f, 0.f, 0.f};
        if (MODE == 1) lse4 = *reinterpret_cast<const floatx4*>(lse_w + (sub * 16 + 4 * c) * 4);
        if (MODE == 0 && track)
            score_rows_max(acc_cur, mask, first + sub * 16 + 4 * c, s_end, lim, p.scale_log2, m_ref, l_run);
        __builtin_amdgcn_sched_barrier(0);
        // Piece i: MFMA i of the next sub-block, the exponent of logit i, the exponential of logit
        // i-1 and the addition of logit i-2: every input was produced a piece earlier, so the wave
        // does not wait on the latency of its own previous instruction.
        float part = 0.f, x_prev = 0.f, y_prev = 0.f;
#pragma unroll
        for (int i = 0; i < 18; ++i) {
            if (has_next && i < 4 * KK) {
                // neighbours in this order are independent: the four accumulators take turns
                const int kk = i / 4, sb = i % 4;
                acc_nxt[sb] = mfma16(af[kk], sf[sb][kk], kk == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc_nxt[sb]);
            }
            if (has_load && i >= 4 && i % 4 == 0 && i / 4 - 1 < KK) {
                // fragment kk of the sub-block after the next one, right after its last reader
                const int kk = i / 4 - 1;
                const int it = (sub + 2) * 16 + r;
                const int swz = (D == 128) ? (it & 15) : ((it >> 1) & 7);
                af[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                    tile + it * ROW_BYTES + (((kk * 4 + c) ^ swz) * 16)));
            }
            if (i >= 2) {                                   // add logit i-2
                const int sb = (i - 2) / 4, e = (i - 2) % 4;
                part = (e == 0) ? y_prev : part + y_prev;
                if (e == 3) {
                    if (MODE == 0) l_run[sb] += part;
                    else col[sb] += part;
                }
            }
            if (i >= 1 && i <= 16) {                        // exponential of logit i-1
                const int sb = (i - 1) / 4, e = (i - 1) % 4;
                y_prev = fast_exp2(x_prev);
                // text query (lim0 + sub*16 + e) - text_pos0 of this tile sees keys <= lim0 + sub*16 + e
                if (MODE == 1 && mask) y_prev = (key_abs[sb] > lim0 + sub * 16 + e) ? 0.f : y_prev;
            }
            if (i < 16) {                                   // exponent of logit i
                const int sb = i / 4, e = i % 4;
                x_prev = (MODE == 0) ? fmaf(acc_cur[sb][e], sc_a, -m_ref[sb])
                                     : fmaf(acc_cur[sb][e], p.scale_log2, -lse4[e]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // (forced inline: as a call the lambda would get every captured array through memory)
    auto tile_body = [&](int stage, int first, int i0, bool mask, bool track) __attribute__((always_inline)) {
        const unsigned char* tile = s_tile + stage * TILE_BYTES;
        const unsigned char* lse_w = s_lse + (stage * 4 + wave) * LSE_BYTES;
        const int lim0 = (MODE == 1) ? p.text_pos0 + i0 + 4 * c : 0;      // i0: the tile's first text query
        bf16x8 af[KK];
        floatx4 acc0[4], acc1[4];
        score_load_a<D>(tile, 0, r, c, af);
        score_mfma<KK>(af, sf, acc0);
        score_load_a<D>(tile, 1, r, c, af);
        step(acc0, acc1, af, tile, lse_w, 0, first, lim0, mask, track, true, true);
        step(acc1, acc0, af, tile, lse_w, 1, first, lim0, mask, track, true, true);
        step(acc0, acc1, af, tile, lse_w, 2, first, lim0, mask, track, true, false);
        step(acc1, acc0, af, tile, lse_w, 3, first, lim0, mask, track, false, false);
    };
    auto compute = [&](int stage, int first, int i0, bool first_tile) __attribute__((always_inline)) {
        // the mask is uniform over the tile (pass A) or the launch (pass B): copies of the
        // straight-line body instead of branches inside it
        if (MODE == 1) {
            if (p.b_needs_mask) tile_body(stage, first, i0, true, false);
            else tile_body(stage, first, i0, false, false);
            return;
        }
        // earliest text query among the workgroup's rows sees keys <= text_pos0
        const bool mask = (first + kScoreTile > s_end) || (first + kScoreTile - 1 > p.text_pos0);
        if (mask) { tile_body(stage, first, i0, true, true); return; }
        if (first_tile) { tile_body(stage, first, i0, false, true); return; }
        // Pass A away from the mask: the maxima are not tracked.  The exponentials are taken
        // against the reference the earlier tiles left; a logit far above it only makes the sum
        // large, and a sum that is no longer a moderate finite number (overflow, or the
        // reference still unset) sends the wave back over the same tile with tracking on.
        float l_save[4];                      // (the references do not move without tracking)
#pragma unroll
        for (int sb = 0; sb < 4; ++sb) l_save[sb] = l_run[sb];
        tile_body(stage, first, i0, false, false);
        bool redo = false;
#pragma unroll
        for (int sb = 0; sb < 4; ++sb) redo = redo || !(l_run[sb] < kSumRedo);
        if (__any(redo)) {
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) l_run[sb] = l_save[sb];
            tile_body(stage, first, i0, false, true);
        }
    };

    // ---- ring: NS-1 tiles in flight while one is consumed; one barrier per tile ----
    // Every wave issues the same number of loads for every tile, in straight-line code: the
    // prologue always fills NS-1 stages and every iteration issues one more tile (past the end of
    // the range the last tile is fetched again into a stage nobody reads), so "tile t has landed"
    // is the constant wait vmcnt <= (NS-2) tiles' worth and nothing makes the compiler add a
    // full drain inside the loop.
    constexpr int LPT = LPW + (MODE == 1 ? 1 : 0);       // loads per wave per tile
    if (n_tiles > 0) {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue_next(s);
        // the stationary fragments (older than the tiles just requested) are in their registers
        __builtin_amdgcn_s_waitcnt(score_vmcnt_imm((NS - 1) * LPT) & ~(15 << 8));
        int t = 0, st_use = 0, st_fill = NS - 1;         // stage consumed / stage refilled this iteration
        int use_i0 = (MODE == 1) ? s_begin % p.l_pad : 0;   // pass B: first text query of the tile consumed
        do {
            __builtin_amdgcn_s_waitcnt(score_vmcnt_imm((NS - 2) * LPT) & ~(15 << 8));
            __asm__ volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            __asm__ volatile("" ::: "memory");
            issue_next(st_fill);
            compute(st_use, s_begin + t * kScoreTile, use_i0, t == 0);
            if (MODE == 1) { use_i0 += kScoreTile; if (use_i0 >= p.l_pad) use_i0 = 0; }
            st_use = (st_use + 1 == NS) ? 0 : st_use + 1;
            st_fill = (st_fill + 1 == NS) ? 0 : st_fill + 1;
        } while (++t < n_tiles);
        __builtin_amdgcn_s_waitcnt(score_vmcnt_imm(0) & ~(15 << 8));   // the surplus loads land before the workgroup ends
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
void score_lse_kernel(const ScoreParams p_launch)
{
    ScoreParams p = p_launch;
    const int row = blockIdx.x * 256 + threadIdx.x, g = blockIdx.y;
    if (row >= p.rows_pad) return;
    if (!score_select_request(p, blockIdx.z)) return;
    float out = INFINITY;                       // padded / keyless rows contribute nothing
    const int gl = row / p.l_pad, i = row % p.l_pad;
    if (row < p.rows && i < p.n_text) {
        if (p.row_lse) {
            out = p.row_lse[(int64_t)i * p.n_q_heads + g * p.group + gl] * kLog2e;
            if (!(out > -INFINITY)) out = INFINITY;
        } else {
            const float2* src = reinterpret_cast<const float2*>(p.part_ml) + ((int64_t)g * p.rows_pad + row) * p.a_splits;
            // online merge of the (max, sum) pairs, eight loads in flight at a time
            float m = kNegBig, l = 0.f;
            for (int s0 = 0; s0 < p.a_splits; s0 += 8) {
                float2 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = (s0 + u < p.a_splits) ? src[s0 + u] : float2{kNegBig, 0.f};
                float mc = m;
#pragma unroll
                for (int u = 0; u < 8; ++u) mc = fmaxf(mc, v[u].x);
                l *= fast_exp2(m - mc);
#pragma unroll
                for (int u = 0; u < 8; ++u) l += v[u].y * fast_exp2(v[u].x - mc);
                m = mc;
            }
            if (l > 0.f) out = m + fast_log2(l);
        }
    }
    p.lse2[(int64_t)g * p.rows_pad + row] = out;
}

__global__ __launch_bounds__(256)
void score_final_kernel(const ScoreParams p_launch)
{
    ScoreParams p = p_launch;
    if (!score_select_request(p, blockIdx.y)) return;           // (layer 0 of request blockIdx.y)
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p.n_video) return;
    float a = 0.f;
    const int parts = p.n_kv_heads * p.b_splits;
    // layer after layer, eight loads in flight at a time; the additions keep the order layer 0, 1, ... and
    // inside a layer s = 0, 1, 2, ...
    for (int layer = 0; layer < p.n_layers; ++layer) {
        const float* cols = p.part_cols + (int64_t)layer * p.batch * p.ws_cols;
        for (int s0 = 0; s0 < parts; s0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = (s0 + u < parts) ? cols[(int64_t)(s0 + u) * p.video_pad + j] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
        }
    }
    a *= p.inv_count;
    p.scores[j] = (p.beta != 0.f ? p.beta * p.scores[j] : 0.f) + a;
}

struct ScorePlan {
    int l_pad, rows, rows_pad, video_pad, key_lo, key_hi, a_splits, a_split_keys, b_splits, b_split_rows;
    size_t off_ml, off_lse, off_cols, total;
};

static ScorePlan score_plan(int batch, int n_text, int n_keys, int video_start, int n_video, int n_q_heads,
                            int n_kv_heads, int head_dim, int norm_mode, int have_row_lse)
{
    ScorePlan s;
    const int group = n_q_heads / n_kv_heads;
    s.l_pad = round_up(n_text > 0 ? n_text : 1, kScoreTile);
    s.rows = group * s.l_pad;
    s.rows_pad = round_up(s.rows, kScoreBlock);
    s.video_pad = round_up(n_video > 0 ? n_video : 1, kScoreBlock);
    s.key_lo = norm_mode ? video_start : 0;
    s.key_hi = norm_mode ? video_start + n_video : n_keys;
    // Workgroups resident per CU: three at head size 128 (168 VGPRs, 51 KB of LDS each), four at
    // 64.  The dispatcher hands a
    // CU its next workgroup as soon as one ends, so a CU that is dealt w workgroups works through
    // them `resident` at a time: its time is about max(w, resident) / resident workgroup
    // lifetimes (below `resident` the CU is under-used, not faster).  Minimise that, ties to the
    // fewer splits (less partial traffic).
    const int resident = head_dim == 128 ? 3 : 4;
    auto best_splits = [&](int blocks, int streamed, int max_splits, int* per_split) {
        int best = 1, best_per = round_up(streamed > 0 ? streamed : 1, kScoreTile);
        long best_cost = -1;
        for (int n = 1; n <= max_splits; ++n) {
            const int per = round_up((streamed + n - 1) / n > 0 ? (streamed + n - 1) / n : 1, kScoreTile);
            const int live = streamed > 0 ? (streamed + per - 1) / per : 1;
            if (live != n) continue;                             // same partition as a smaller n
            const long wgs = (long)blocks * live;
            const long per_cu = (wgs + kNumCu - 1) / kNumCu;
            // +2 tiles: a workgroup's fixed cost (stationary fragments, ring fill); + live: fewer splits on ties
            const long cost = (per_cu > resident ? per_cu : resident) * (per / kScoreTile + 2) * 64 / resident + live;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = live; best_per = per; }
        }
        *per_split = best_per;
        return best;
    };
    const int dom = s.key_hi - s.key_lo;
    const int blocks_a = (s.rows_pad / kScoreBlock) * n_kv_heads * batch;
    s.a_splits = best_splits(blocks_a, dom, kMaxSplitsA, &s.a_split_keys);
    const int blocks_b = (s.video_pad / kScoreBlock) * n_kv_heads * batch;
    s.b_splits = best_splits(blocks_b, s.rows, kMaxSplitsB, &s.b_split_rows);
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

extern "C" size_t specvlm_score_layers_workspace_bytes(int n_layers, int batch, int n_text, int n_keys, int n_video,
                                                       int n_q_heads, int n_kv_heads, int head_dim,
                                                       int have_row_lse)
{
    if (n_layers < 1 || batch < 1 || (int64_t)n_layers * batch > 65535 || n_text < 0 || n_keys < 0 || n_video < 0 ||
        n_video > n_keys || n_kv_heads <= 0 || n_q_heads <= 0 || n_q_heads % n_kv_heads)
        return 0;
    // every (layer, request) has its own slice, sized by the plan of the maxima; the split plan
    // depends on the normalisation domain: size for the larger one
    const int units = n_layers * batch;
    const ScorePlan a = score_plan(units, n_text, n_keys, 0, n_video, n_q_heads, n_kv_heads, head_dim, 0, have_row_lse);
    const ScorePlan b = score_plan(units, n_text, n_keys, 0, n_video, n_q_heads, n_kv_heads, head_dim, 1, have_row_lse);
    return (size_t)units * (a.total > b.total ? a.total : b.total);
}

extern "C" size_t specvlm_score_workspace_bytes(int batch, int n_text, int n_keys, int n_video,
                                                int n_q_heads, int n_kv_heads, int head_dim,
                                                int have_row_lse)
{
    return specvlm_score_layers_workspace_bytes(1, batch, n_text, n_keys, n_video, n_q_heads, n_kv_heads, head_dim,
                                                have_row_lse);
}

static int score_impl(
    const void* q_text,  int64_t q_layer_stride, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k_cache, int64_t k_layer_stride, int64_t k_tok_stride, int64_t k_head_stride, int n_layers,
    const int32_t* cu_text, const int32_t* cu_keys, const int32_t* cu_video, int batch,
    int n_text, int n_keys, int video_start, int n_video, int text_pos0,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    int norm_mode, const float* row_lse, int64_t lse_layer_stride, float beta, float* scores,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_layers < 0) return SPECVLM_EINVAL;
    if ((q_layer_stride | k_layer_stride) & 7) return SPECVLM_EUNSUPPORTED;
    if (batch < 0 || text_pos0 < -1) return SPECVLM_EINVAL;
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads) return SPECVLM_EINVAL;
    if (norm_mode != 0 && norm_mode != 1) return SPECVLM_EINVAL;
    if (!(softmax_scale >= 0.f) || !(softmax_scale < INFINITY)) return SPECVLM_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SPECVLM_EUNSUPPORTED;
    if ((q_tok_stride | q_head_stride | k_tok_stride | k_head_stride) & 7) return SPECVLM_EUNSUPPORTED;
    // a lane's byte offset inside a 64-vector tile is kept in 32 bits
    if (q_tok_stride < 0 || k_tok_stride < 0 || q_tok_stride >= (1 << 24) || k_tok_stride >= (1 << 24))
        return SPECVLM_EUNSUPPORTED;
    if (batch == 0) return SPECVLM_OK;
    const bool ragged = cu_text || cu_keys || cu_video;
    if (ragged && !(cu_text && cu_keys && cu_video)) return SPECVLM_EINVAL;
    if (!ragged && batch != 1) return SPECVLM_EINVAL;
    if ((int64_t)batch * (n_layers > 0 ? n_layers : 1) > 65535) return SPECVLM_EUNSUPPORTED;
    if (n_text < 0 || n_keys < 0 || video_start < 0 || n_video < 0) return SPECVLM_EINVAL;
    if ((int64_t)video_start + n_video > n_keys) return SPECVLM_EINVAL;
    if (!ragged) {
        if (text_pos0 < 0) text_pos0 = n_keys - n_text;       // -1: the text queries are the last keys
        if (text_pos0 < 0) return SPECVLM_EINVAL;
    }
    if (n_video == 0) return SPECVLM_OK;
    if (!scores) return SPECVLM_EINVAL;
    if (n_text > 0 && n_layers > 0 && (!q_text || !k_cache)) return SPECVLM_EINVAL;
    if (((uintptr_t)q_text | (uintptr_t)k_cache) & 15) return SPECVLM_EUNSUPPORTED;

    // One plan for all layers and the whole batch, made from the maxima (the host does not know the
    // requests' own sizes); a request's kernels find their real sizes in the cu arrays on the device.
    // Without layers only beta applies (the sum over layers is empty).
    const int units = batch * n_layers;                 // (layer, request) pairs: one workspace slice each
    const ScorePlan plan = score_plan(units > 0 ? units : 1, n_text, n_keys, video_start, n_video, n_q_heads,
                                      n_kv_heads, head_dim, norm_mode, row_lse != nullptr);
    if (units > 0 && (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < (size_t)units * plan.total))
        return SPECVLM_EWORKSPACE;
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
    // workspace: [layers x batch] slices of each of the three arrays
    const size_t n_ml = row_lse ? 0 : (size_t)n_kv_heads * plan.rows_pad * plan.a_splits * 2;
    const size_t n_lse = (size_t)n_kv_heads * plan.rows_pad;
    const size_t n_cols = (size_t)n_kv_heads * plan.b_splits * plan.video_pad;
    char* ws = (char*)workspace;
    p.part_ml = (float*)ws;  ws += align256(units * n_ml * sizeof(float));
    p.lse2 = (float*)ws;     ws += align256(units * n_lse * sizeof(float));
    p.part_cols = (float*)ws;
    p.ws_ml = (int64_t)n_ml; p.ws_lse = (int64_t)n_lse; p.ws_cols = (int64_t)n_cols;
    p.row_lse = row_lse;
    p.beta = beta;
    p.inv_count = (n_text > 0) ? 1.f / ((float)n_q_heads * (float)n_text) : 0.f;
    p.scores = scores;
    p.cu_text = cu_text; p.cu_keys = cu_keys; p.cu_video = cu_video;
    p.batch = batch; p.norm_mode = norm_mode;
    p.n_layers = n_layers; p.q_layer = q_layer_stride; p.k_layer = k_layer_stride; p.lse_layer = lse_layer_stride;
    hipStream_t s = (hipStream_t)stream;

    if (n_text > 0 && n_layers > 0) {
        if ((int64_t)(plan.rows_pad / kScoreBlock) * n_kv_heads * plan.a_splits * units > 0x7fffff00ll ||
            (int64_t)(plan.video_pad / kScoreBlock) * n_kv_heads * plan.b_splits * units > 0x7fffff00ll)
            return SPECVLM_EUNSUPPORTED;
        if (!row_lse && p.key_hi > p.key_lo) {
            dim3 grid(round_up((plan.rows_pad / kScoreBlock) * n_kv_heads * plan.a_splits * units, kNumXcd));
            if (head_dim == 128) hipLaunchKernelGGL((score_sweep_kernel<128, 0>), grid, dim3(256), 0, s, p);
            else                 hipLaunchKernelGGL((score_sweep_kernel<64, 0>), grid, dim3(256), 0, s, p);
        }
        hipLaunchKernelGGL(score_lse_kernel, dim3(plan.rows_pad / 256, n_kv_heads, units), dim3(256), 0, s, p);
        dim3 grid(round_up((plan.video_pad / kScoreBlock) * n_kv_heads * plan.b_splits * units, kNumXcd));
        if (head_dim == 128) hipLaunchKernelGGL((score_sweep_kernel<128, 1>), grid, dim3(256), 0, s, p);
        else                 hipLaunchKernelGGL((score_sweep_kernel<64, 1>), grid, dim3(256), 0, s, p);
    } else {
        p.b_splits = 0;          // no language queries in the whole batch: the mean is empty, only beta applies
    }
    hipLaunchKernelGGL(score_final_kernel, dim3((n_video + 255) / 256, batch), dim3(256), 0, s, p);
    return launch_status();
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
    return score_impl(q_text, 0, q_tok_stride, q_head_stride, k_cache, 0, k_tok_stride, k_head_stride, 1,
                      cu_text, cu_keys, cu_video, batch, n_text, n_keys, video_start, n_video, text_pos0,
                      n_q_heads, n_kv_heads, head_dim, softmax_scale, norm_mode, row_lse, 0, beta, scores,
                      workspace, workspace_bytes, stream);
}

extern "C" int specvlm_score_layers(
    const void* q_text,  int64_t q_layer_stride, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k_cache, int64_t k_layer_stride, int64_t k_tok_stride, int64_t k_head_stride, int n_layers,
    const int32_t* cu_text, const int32_t* cu_keys, const int32_t* cu_video, int batch,
    int n_text, int n_keys, int video_start, int n_video, int text_pos0,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    int norm_mode, const float* row_lse, int64_t row_lse_layer_stride, float beta, float* scores,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return score_impl(q_text, q_layer_stride, q_tok_stride, q_head_stride, k_cache, k_layer_stride, k_tok_stride,
                      k_head_stride, n_layers, cu_text, cu_keys, cu_video, batch, n_text, n_keys, video_start,
                      n_video, text_pos0, n_q_heads, n_kv_heads, head_dim, softmax_scale, norm_mode, row_lse,
                      row_lse_layer_stride, beta, scores, workspace, workspace_bytes, stream);
}
