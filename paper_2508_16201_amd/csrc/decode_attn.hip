// specvlm_decode_attn: grouped-query softmax attention of a short query block
// (1 query for plain decode, gamma+1 for parallel verification; Sec. 2.1 of the
// paper) over a long bf16 KV cache, in split-K (flash-decode) form for gfx950.
//
// Work decomposition
//   One workgroup (4 waves) owns one (request, kv head, key split).  All
//   G*q_len query rows that share the kv head are packed into the MFMA "row"
//   dimension (up to 4 blocks of 16 rows), so every K/V byte is read from HBM
//   exactly once.  Inside the workgroup the split's 32-key tiles are dealt
//   round-robin to the 4 waves; each wave runs an independent online softmax
//   and the four partial results are merged through LDS at the end.
//
// MFMA formulation (v_mfma_f32_16x16x32_bf16, lane = 16*c + r)
//   S^T = K Q^T : A = K tile (rows = 16 keys, contraction = d), B = Q^T.  The
//     result puts query row r in lane column r and keys 4c..4c+3 in the four
//     accumulator registers, so all softmax statistics of a row live in the
//     lanes r, r+16, r+32, r+48.
//   O^T = V^T P^T : B = P^T is exactly what the lane already holds (row r, the
//     8 keys {4c..4c+3} of both 16-key sub-tiles); A = V^T needs, per lane, 8
//     keys x 1 value column.  Each lane loads 8 (d=128) contiguous value
//     columns of its 8 keys (a full 256-byte row per 16 lanes) and an in-lane
//     16-bit transpose (v_perm) forms the operands.  The contraction order over
//     keys and the column order of O are permutations fixed by this layout, so
//     neither K nor V ever goes through LDS.
//   O^T keeps row r in lane column r as well: rescaling by the running max is a
//     per-lane multiply.
#include "common.h"

namespace specvlm {

struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    __bf16* out;
    float* lse;
    int64_t q_tok, q_head, kv_tok, kv_head;
    const int32_t* cu_q;
    const int32_t* cu_kv;
    int batch, q_len, kv_len, n_q_heads, n_kv_heads, group;
    float scale_log2;        // softmax_scale * log2(e)
    int num_splits, split_keys;
    float* part_o;           // [batch*H_kv][num_splits][rows_pad][D] unnormalised partial outputs
    float* part_ml;          // [batch*H_kv][num_splits][rows_pad][2] (running max in log2 units, sum)
    int rows_pad;
    int n_work, n_work_padded;
};

constexpr int kTileKeys = 32;
constexpr int kAttnWaves = 4;
constexpr int kMaxSplits = 256;

template <int D> struct ValueVec;
template <> struct ValueVec<128> { typedef u32x4 type; };
template <> struct ValueVec<64>  { typedef u32x2 type; };

template <int D, int MB>
__global__ __launch_bounds__(kAttnWaves * kWave)
void attn_split_kernel(const AttnParams p)
{
    constexpr int DJ = D / 16;          // value columns per lane (8 or 4)
    constexpr int KK = D / 32;          // MFMA steps over the head dimension
    constexpr int LDS_STRIDE = D + 4;
    typedef typename ValueVec<D>::type vvec_t;

    const int vid = xcd_logical_id(blockIdx.x, p.n_work_padded);
    if (vid >= p.n_work) return;
    const int split = vid % p.num_splits;
    const int bh = vid / p.num_splits;
    const int b = bh / p.n_kv_heads, g = bh % p.n_kv_heads;

    int q0 = 0, ql = p.q_len, kv0 = 0, kvl = p.kv_len;
    if (p.cu_q) { q0 = p.cu_q[b]; ql = p.cu_q[b + 1] - q0; }
    if (p.cu_kv) { kv0 = p.cu_kv[b]; kvl = p.cu_kv[b + 1] - kv0; }
    if (ql <= 0 || kvl < ql) return;
    const int k_begin = split * p.split_keys;
    if (k_begin >= kvl) return;                     // the merge reads only the live splits
    const int k_end = min(kvl, k_begin + p.split_keys);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, c = lane >> 4;
    const int n_rows = p.group * ql;                // live query rows of this kv head

    // ---- Q fragments (B operand of S^T) staged in LDS in fragment order: the
    // waves re-read them per tile instead of pinning MB*KK*4 registers each ----
    extern __shared__ __align__(16) float smem[];
    u32x4* q_lds = reinterpret_cast<u32x4*>(smem);        // [MB][KK][64 lanes]
    int last_key[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = mb * 16 + r;
        const bool live = row < n_rows;
        const int t = live ? row / p.group : 0;
        const int h = g * p.group + (live ? row % p.group : 0);
        last_key[mb] = kvl - ql + t;
        const __bf16* qp = p.q + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head + c * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (((mb * KK + kk) & (kAttnWaves - 1)) != wave) continue;
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (live) raw = *reinterpret_cast<const u32x4*>(qp + kk * 32);
            q_lds[(mb * KK + kk) * kWave + lane] = raw;
        }
    }
    __syncthreads();

    // Uniform (scalar) request/head base plus 32-bit per-lane byte offsets.
    const char* kbase = reinterpret_cast<const char*>(p.k + (int64_t)kv0 * p.kv_tok + (int64_t)g * p.kv_head);
    const char* vbase = reinterpret_cast<const char*>(p.v + (int64_t)kv0 * p.kv_tok + (int64_t)g * p.kv_head);
    const uint32_t tok_bytes = (uint32_t)p.kv_tok * 2u;
    const uint32_t k_lane = (uint32_t)c * 16u, v_lane = (uint32_t)r * (DJ * 2u);

    float m_run[MB], l_run[MB];
    floatx4 o_acc[MB][DJ];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -INFINITY;
        l_run[mb] = 0.f;
#pragma unroll
        for (int j = 0; j < DJ; ++j) o_acc[mb][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // Keys of a tile as seen by this lane: sub-tile 0 rows r (K operand) and, for
    // the values / probabilities, keys 4c+i (i<4) and 16+4c+(i-4) (i>=4).
    auto load_tile = [&](int base, u32x4 (&kr)[2][KK], vvec_t (&vr)[8]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const uint32_t key = (uint32_t)min(base + kt * 16 + r, kvl - 1);
            const char* kp = kbase + (key * tok_bytes + k_lane);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                kr[kt][kk] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + kk * 64));
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t key = (uint32_t)min(base + (i < 4 ? 4 * c + i : 16 + 4 * c + (i - 4)), kvl - 1);
            vr[i] = __builtin_nontemporal_load(
                reinterpret_cast<const vvec_t*>(vbase + (key * tok_bytes + v_lane)));
        }
    };

    auto compute_tile = [&](int base, const u32x4 (&kr)[2][KK], const vvec_t (&vr)[8]) {
        const bool need_mask = (base + kTileKeys > k_end) || (base + kTileKeys - 1 > kvl - ql);
        __asm__ volatile("" ::: "memory");       // keep the Q fragment reads inside the loop
        bf16x8 pf[MB];
        bool rescale = false;
        float alpha[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 qf = __builtin_bit_cast(bf16x8, q_lds[(mb * KK + kk) * kWave + lane]);
                s0 = mfma16(__builtin_bit_cast(bf16x8, kr[0][kk]), qf, s0);
                s1 = mfma16(__builtin_bit_cast(bf16x8, kr[1][kk]), qf, s1);
            }
            float s[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { s[i] = s0[i] * p.scale_log2; s[4 + i] = s1[i] * p.scale_log2; }
            if (need_mask) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int key = base + (i < 4 ? 4 * c + i : 16 + 4 * c + (i - 4));
                    if (key >= k_end || key > last_key[mb]) s[i] = -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                             fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[mb], mx);
            const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[mb] = fast_exp2(m_run[mb] - m_ref);
            rescale = rescale || (m_new != m_run[mb]);
            m_run[mb] = m_new;
            floatx8 pv;
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { pv[i] = fast_exp2(s[i] - m_ref); psum += pv[i]; }
            l_run[mb] = l_run[mb] * alpha[mb] + psum;
            pf[mb] = __builtin_convertvector(pv, bf16x8);
        }
        if (__any(rescale)) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < DJ; ++j) o_acc[mb][j] *= alpha[mb];
        }
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            // in-lane transpose: value column j of the lane's 8 keys
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            u32x4 vt;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr)
                vt[pr] = __builtin_amdgcn_perm(vr[2 * pr + 1][j >> 1], vr[2 * pr][j >> 1], sel);
            const bf16x8 va = __builtin_bit_cast(bf16x8, vt);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) o_acc[mb][j] = mfma16(va, pf[mb], o_acc[mb][j]);
        }
    };

    // ---- stream the split's tiles, one tile of prefetch per wave ----
    const int n_tiles = (k_end - k_begin + kTileKeys - 1) / kTileKeys;
    {
        u32x4 ka[2][KK], kb[2][KK];
        vvec_t va[8], vb[8];
        int ti = wave;
        if (ti < n_tiles) load_tile(k_begin + ti * kTileKeys, ka, va);
        while (ti < n_tiles) {
            int tn = ti + kAttnWaves;
            if (tn < n_tiles) load_tile(k_begin + tn * kTileKeys, kb, vb);
            compute_tile(k_begin + ti * kTileKeys, ka, va);
            ti = tn;
            if (ti >= n_tiles) break;
            tn = ti + kAttnWaves;
            if (tn < n_tiles) load_tile(k_begin + tn * kTileKeys, ka, va);
            compute_tile(k_begin + ti * kTileKeys, kb, vb);
            ti = tn;
        }
    }

    // ---- merge the four waves through LDS (reusing the Q staging area) ----
    __syncthreads();
    float* sm_m = smem;                              // [4][MB*16]
    float* sm_l = sm_m + kAttnWaves * MB * 16;       // [4][MB*16]
    float* sm_o = sm_l + kAttnWaves * MB * 16;       // [2][MB*16][LDS_STRIDE]
    constexpr int OBUF = MB * 16 * LDS_STRIDE;

#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        l_run[mb] += __shfl_xor(l_run[mb], 16);
        l_run[mb] += __shfl_xor(l_run[mb], 32);
        if (c == 0) sm_m[wave * MB * 16 + mb * 16 + r] = m_run[mb];
    }
    __syncthreads();
    float m_all[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        float mm = sm_m[mb * 16 + r];
#pragma unroll
        for (int w = 1; w < kAttnWaves; ++w) mm = fmaxf(mm, sm_m[w * MB * 16 + mb * 16 + r]);
        m_all[mb] = mm;
        const float f = fast_exp2(m_run[mb] - ((mm == -INFINITY) ? 0.f : mm));
        l_run[mb] *= f;
#pragma unroll
        for (int j = 0; j < DJ; ++j) o_acc[mb][j] *= f;
        if (c == 0) sm_l[wave * MB * 16 + mb * 16 + r] = l_run[mb];
    }
    // lane (r, c) holds columns [4*DJ*c, 4*DJ*(c+1)) of row r: column (4c+i)*DJ + j
    auto lds_store = [&](float* buf) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < DJ / 4; ++jj) {
                    floatx4 x = {o_acc[mb][4 * jj][i], o_acc[mb][4 * jj + 1][i],
                                 o_acc[mb][4 * jj + 2][i], o_acc[mb][4 * jj + 3][i]};
                    *reinterpret_cast<floatx4*>(buf + (mb * 16 + r) * LDS_STRIDE +
                                                (4 * c + i) * DJ + 4 * jj) = x;
                }
    };
    auto lds_add = [&](const float* buf) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < DJ / 4; ++jj) {
                    const floatx4 x = *reinterpret_cast<const floatx4*>(
                        buf + (mb * 16 + r) * LDS_STRIDE + (4 * c + i) * DJ + 4 * jj);
#pragma unroll
                    for (int e = 0; e < 4; ++e) o_acc[mb][4 * jj + e][i] += x[e];
                }
    };
    if (wave & 1) lds_store(sm_o + (wave >> 1) * OBUF);
    __syncthreads();
    if (!(wave & 1)) lds_add(sm_o + (wave >> 1) * OBUF);
    __syncthreads();
    if (wave == 2) lds_store(sm_o);
    __syncthreads();
    if (wave != 0) return;
    lds_add(sm_o);

    const bool final_out = (p.num_splits == 1);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = mb * 16 + r;
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) l_all += sm_l[w * MB * 16 + row];
        if (final_out) {
            if (row >= n_rows) continue;
            const int t = row / p.group, h = g * p.group + row % p.group;
            const float inv = 1.f / l_all;
            __bf16* op = p.out + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < DJ / 4; ++jj) {
                    floatx4 x = {o_acc[mb][4 * jj][i], o_acc[mb][4 * jj + 1][i],
                                 o_acc[mb][4 * jj + 2][i], o_acc[mb][4 * jj + 3][i]};
                    x *= inv;
                    const bf16x4 y = __builtin_convertvector(x, bf16x4);
                    *reinterpret_cast<bf16x4*>(op + (4 * c + i) * DJ + 4 * jj) = y;
                }
            if (p.lse && c == 0)
                p.lse[(int64_t)(q0 + t) * p.n_q_heads + h] = (m_all[mb] + fast_log2(l_all)) * kLn2;
        } else {
            const int64_t slot = ((int64_t)bh * p.num_splits + split) * p.rows_pad + row;
            float* po = p.part_o + slot * D;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < DJ / 4; ++jj) {
                    floatx4 x = {o_acc[mb][4 * jj][i], o_acc[mb][4 * jj + 1][i],
                                 o_acc[mb][4 * jj + 2][i], o_acc[mb][4 * jj + 3][i]};
                    *reinterpret_cast<floatx4*>(po + (4 * c + i) * DJ + 4 * jj) = x;
                }
            if (c == 0) {
                p.part_ml[slot * 2] = m_all[mb];
                p.part_ml[slot * 2 + 1] = l_all;
            }
        }
    }
}

// Merge of the split partials: o = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s.
// One workgroup per (kv head, query row).  All loads of a phase are independent
// (one split per thread for the statistics, splits strided over thread groups
// for the outputs), so the kernel costs a few memory round trips, not one per split.
template <int D>
__global__ __launch_bounds__(256)
void attn_merge_kernel(const AttnParams p)
{
    constexpr int TPR = D / 4;                       // threads that cover one row of D columns
    constexpr int GROUPS = 256 / TPR;                // split groups working in parallel
    __shared__ float s_w[kMaxSplits];
    __shared__ float s_red[8];
    __shared__ __align__(16) float s_acc[GROUPS][D];
    const int row = blockIdx.x, bh = blockIdx.y;
    const int b = bh / p.n_kv_heads, g = bh % p.n_kv_heads;
    int q0 = 0, ql = p.q_len, kvl = p.kv_len;
    if (p.cu_q) { q0 = p.cu_q[b]; ql = p.cu_q[b + 1] - q0; }
    if (p.cu_kv) { kvl = p.cu_kv[b + 1] - p.cu_kv[b]; }
    if (ql <= 0 || kvl < ql || row >= p.group * ql) return;
    const int live = min(p.num_splits, (kvl + p.split_keys - 1) / p.split_keys);
    const int64_t slot0 = (int64_t)bh * p.num_splits * p.rows_pad + row;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // phase 1: one split per thread -> global max, weights, total sum
    float m_s = -INFINITY, l_s = 0.f;
    if (tid < live) {
        const float* ml = p.part_ml + (slot0 + (int64_t)tid * p.rows_pad) * 2;
        m_s = ml[0]; l_s = ml[1];
    }
    float m = m_s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    const float m_ref = (m == -INFINITY) ? 0.f : m;
    const float w_s = (tid < live) ? fast_exp2(m_s - m_ref) : 0.f;
    s_w[tid] = w_s;
    float l = w_s * l_s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off);
    if (lane == 0) s_red[4 + wave] = l;
    __syncthreads();
    l = (s_red[4] + s_red[5]) + (s_red[6] + s_red[7]);

    // phase 2: group `grp` accumulates splits grp, grp+GROUPS, ... for 4 columns
    const int grp = tid / TPR, col = (tid % TPR) * 4;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = grp; s < live; s += GROUPS)
        acc += s_w[s] * *reinterpret_cast<const floatx4*>(
                            p.part_o + (slot0 + (int64_t)s * p.rows_pad) * D + col);
    *reinterpret_cast<floatx4*>(&s_acc[grp][col]) = acc;
    __syncthreads();
    if (grp != 0) return;
#pragma unroll
    for (int gg = 1; gg < GROUPS; ++gg) acc += *reinterpret_cast<const floatx4*>(&s_acc[gg][col]);
    acc *= 1.f / l;
    const int t = row / p.group, h = g * p.group + row % p.group;
    __bf16* op = p.out + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head + col;
    *reinterpret_cast<bf16x4*>(op) = __builtin_convertvector(acc, bf16x4);
    if (p.lse && col == 0)
        p.lse[(int64_t)(q0 + t) * p.n_q_heads + h] = (m + fast_log2(l)) * kLn2;
}

static int choose_splits(int batch, int kv_len, int n_kv_heads, int num_splits)
{
    const int max_by_len = (kv_len + kAttnWaves * kTileKeys - 1) / (kAttnWaves * kTileKeys);
    int s = num_splits;
    if (s <= 0) {
        const int heads = batch * n_kv_heads;
        s = (kNumCu + heads - 1) / heads;
    }
    if (s > max_by_len) s = max_by_len;
    if (s > kMaxSplits) s = kMaxSplits;
    if (s < 1) s = 1;
    return s;
}

static size_t attn_lds_bytes(int mb, int d)
{
    const size_t merge = sizeof(float) * (size_t)(2 * kAttnWaves * mb * 16 + 2 * mb * 16 * (d + 4));
    const size_t qstage = (size_t)mb * (d / 32) * kWave * 16;
    return merge > qstage ? merge : qstage;
}

template <int D, int MB>
static int launch_attn(const AttnParams& p, hipStream_t stream)
{
    const size_t lds = attn_lds_bytes(MB, D);
    if (lds > 64 * 1024) {
        static bool raised = false;
        if (!raised) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_split_kernel<D, MB>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                return SPECVLM_ELAUNCH;
            raised = true;
        }
    }
    hipLaunchKernelGGL((attn_split_kernel<D, MB>), dim3(p.n_work_padded), dim3(kAttnWaves * kWave),
                       lds, stream, p);
    return launch_status();
}

template <int D>
static int launch_attn_d(const AttnParams& p, int mb, hipStream_t stream)
{
    switch (mb) {
        case 1: return launch_attn<D, 1>(p, stream);
        case 2: return launch_attn<D, 2>(p, stream);
        case 3: return launch_attn<D, 3>(p, stream);
        case 4: return launch_attn<D, 4>(p, stream);
    }
    return SPECVLM_EUNSUPPORTED;
}

}  // namespace specvlm

using namespace specvlm;

extern "C" size_t specvlm_decode_attn_workspace_bytes(int batch, int q_len, int kv_len,
                                                      int n_q_heads, int n_kv_heads, int head_dim,
                                                      int num_splits)
{
    if (batch <= 0 || q_len <= 0 || kv_len <= 0 || n_kv_heads <= 0 || n_q_heads <= 0 ||
        n_q_heads % n_kv_heads || (head_dim != 64 && head_dim != 128))
        return 0;
    const int rows = (n_q_heads / n_kv_heads) * q_len;
    if (rows > 64) return 0;
    const int rows_pad = round_up(rows, 16);
    const int splits = choose_splits(batch, kv_len, n_kv_heads, num_splits);
    if (splits == 1) return 256;
    const size_t slots = (size_t)batch * n_kv_heads * splits * rows_pad;
    return align256(slots * head_dim * sizeof(float)) + align256(slots * 2 * sizeof(float));
}

extern "C" int specvlm_decode_attn(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    void* out, float* lse, int num_splits,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch < 0 || q_len < 0 || kv_len < 0 || n_q_heads <= 0 || n_kv_heads <= 0) return SPECVLM_EINVAL;
    if (n_q_heads % n_kv_heads) return SPECVLM_EINVAL;
    if ((cu_q == nullptr) != (cu_kv == nullptr)) return SPECVLM_EINVAL;
    if (!cu_q && batch > 1) return SPECVLM_EINVAL;
    if (!(softmax_scale >= 0.f) || !(softmax_scale < INFINITY)) return SPECVLM_EINVAL;
    if (num_splits < 0) return SPECVLM_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SPECVLM_EUNSUPPORTED;
    if (batch == 0 || q_len == 0) return SPECVLM_OK;
    if (q_len > kv_len) return SPECVLM_EINVAL;
    if (!q || !k || !v || !out) return SPECVLM_EINVAL;
    if ((q_tok_stride | q_head_stride | kv_tok_stride | kv_head_stride) & 7) return SPECVLM_EUNSUPPORTED;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return SPECVLM_EUNSUPPORTED;
    const int group = n_q_heads / n_kv_heads;
    const int rows = group * q_len;
    if (rows > 64) return SPECVLM_EUNSUPPORTED;
    // per-lane key offsets are 32-bit byte offsets from the request's first row
    if (kv_tok_stride <= 0 || (int64_t)kv_len * kv_tok_stride * 2 >= ((int64_t)1 << 32))
        return SPECVLM_EUNSUPPORTED;
    const int mb = (rows + 15) / 16;

    AttnParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.out = (__bf16*)out; p.lse = lse;
    p.q_tok = q_tok_stride; p.q_head = q_head_stride;
    p.kv_tok = kv_tok_stride; p.kv_head = kv_head_stride;
    p.cu_q = cu_q; p.cu_kv = cu_kv;
    p.batch = batch; p.q_len = q_len; p.kv_len = kv_len;
    p.n_q_heads = n_q_heads; p.n_kv_heads = n_kv_heads; p.group = group;
    p.scale_log2 = softmax_scale * kLog2e;
    p.num_splits = choose_splits(batch, kv_len, n_kv_heads, num_splits);
    p.split_keys = (kv_len + p.num_splits - 1) / p.num_splits;
    p.rows_pad = mb * 16;
    p.n_work = batch * n_kv_heads * p.num_splits;
    p.n_work_padded = round_up(p.n_work, kNumXcd);
    p.part_o = nullptr; p.part_ml = nullptr;
    if (p.num_splits > 1) {
        const size_t need = specvlm_decode_attn_workspace_bytes(batch, q_len, kv_len, n_q_heads,
                                                                n_kv_heads, head_dim, p.num_splits);
        if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SPECVLM_EWORKSPACE;
        const size_t slots = (size_t)batch * n_kv_heads * p.num_splits * p.rows_pad;
        p.part_o = (float*)workspace;
        p.part_ml = (float*)((char*)workspace + align256(slots * head_dim * sizeof(float)));
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = head_dim == 128 ? launch_attn_d<128>(p, mb, s) : launch_attn_d<64>(p, mb, s);
    if (rc != SPECVLM_OK) return rc;
    if (p.num_splits > 1) {
        dim3 grid(rows, batch * n_kv_heads);
        if (head_dim == 128) hipLaunchKernelGGL(attn_merge_kernel<128>, grid, dim3(256), 0, s, p);
        else                 hipLaunchKernelGGL(attn_merge_kernel<64>, grid, dim3(256), 0, s, p);
        rc = launch_status();
    }
    return rc;
}
