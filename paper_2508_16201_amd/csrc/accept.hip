// specvlm_accept: which drafted tokens survive the target's verification
// (Sec. 2.1; greedy target decoding as in App. A, or the rejection-sampling rule
// of speculative sampling that keeps the target's output distribution).
//
// Pass 1 (many workgroups): per (request, row, vocab chunk) partial statistics
//   -- argmax with lowest-index ties for greedy; running (max, sum exp) of
//   logit/T for the target rows and the draft rows for sampling.
// Pass 2, greedy (one wave per request): merge the partials and walk the gamma tests in order.
// Pass 2, sampling (many workgroups): every workgroup merges the partials and repeats the gamma
//   accept tests (a few loads), so all agree on the first rejected position n; each then sums the
//   mass of the residual max(p - q, 0) at row n (of p when every draft survived) over its chunk.
// Pass 3, sampling (one workgroup per request): inverse CDF over the chunk masses, then inside
//   the owning chunk over its waves, then inside the owning wave's tokens.
#include "common.h"

namespace specvlm {

constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kAccChunk = 8192;        // vocab entries per pass-1 workgroup
constexpr int kAccPerThread = kAccChunk / 256;   // of which each of the 256 threads takes this many

struct AcceptParams {
    const float* target;      // [batch, gamma+1, vocab]
    const float* draft;       // [batch, gamma, vocab] or null
    const int32_t* tokens;    // [batch, gamma]
    const float* uniforms;    // [batch, gamma+1] or null
    int batch, gamma, vocab, n_chunks;
    float inv_t_log2;         // log2(e) / temperature
    int32_t* n_accepted;
    int32_t* out_tokens;
    float* part_val;          // [batch][rows][n_chunks]   max
    float* part_aux;          // [batch][rows][n_chunks]   sum exp (sampling) / argmax index bits (greedy)
    float* norm;              // sampling: [batch][rows][2] merged (max, sum exp) of every row
    float* chunk_mass;        // sampling: [batch][n_chunks] residual (or target) mass of row n per chunk
    int32_t* n_rej;           // sampling: [batch] first rejected position n (gamma if none)
};

__device__ __forceinline__ void argmax_merge(float& bv, int& bi, float v, int i)
{
    // larger value wins; equal values: lower index wins.  (i < 0 = empty)
    if (i >= 0 && (bi < 0 || v > bv || (v == bv && i < bi))) { bv = v; bi = i; }
}

// ---------------------------------------------------------------- greedy ----
__global__ __launch_bounds__(256)
void accept_argmax_partial(const AcceptParams p)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const int chunk = blockIdx.x, row = blockIdx.y, b = blockIdx.z;
    const float* x = p.target + ((int64_t)b * (p.gamma + 1) + row) * p.vocab;
    const int lo = chunk * kAccChunk, hi = min(p.vocab, lo + kAccChunk);
    // the thread's whole share is requested before the first value is looked at: one round trip
    float y[kAccPerThread];
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) {
        const int v = lo + j * 256 + threadIdx.x;
        y[j] = v < hi ? x[v] : 0.f;
    }
    float bv = 0.f; int bi = -1;
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) {
        const int v = lo + j * 256 + threadIdx.x;
        if (v < hi && (bi < 0 || y[j] > bv)) { bv = y[j]; bi = v; }     // ascending v: first maximum is kept
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        argmax_merge(bv, bi, ov, oi);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) argmax_merge(bv, bi, s_v[w], s_i[w]);
        const int64_t slot = ((int64_t)b * (p.gamma + 1) + row) * p.n_chunks + chunk;
        p.part_val[slot] = bv;
        p.part_aux[slot] = __int_as_float(bi);
    }
}

__global__ __launch_bounds__(64)
void accept_greedy_final(const AcceptParams p)
{
    // one wave per request; lane i merges the partials of row i and holds drafted token i
    // (gamma <= 64), the first mismatch is found by a ballot and every lane writes its own output
    const int b = blockIdx.x, lane = threadIdx.x;
    __shared__ int s_t[65];
    const int32_t* x = p.tokens + (int64_t)b * p.gamma;
    const int drafted = lane < p.gamma ? x[lane] : -1;           // (in flight while the partials are merged)
    for (int row = lane; row <= p.gamma; row += 64) {
        float bv = 0.f; int bi = -1;
        const int64_t slot = ((int64_t)b * (p.gamma + 1) + row) * p.n_chunks;
        for (int c0 = 0; c0 < p.n_chunks; c0 += 8) {             // eight chunks' loads in flight at a time
            float pv[8]; int pi[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = c0 + j < p.n_chunks;
                pv[j] = in ? p.part_val[slot + c0 + j] : 0.f;
                pi[j] = in ? __float_as_int(p.part_aux[slot + c0 + j]) : -1;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) argmax_merge(bv, bi, pv[j], pi[j]);
        }
        s_t[row] = bi;
    }
    __syncthreads();
    const uint64_t mismatch = __ballot(lane < p.gamma && drafted != s_t[lane]);
    const int n = mismatch ? __ffsll((long long)mismatch) - 1 : p.gamma;
    int32_t* out = p.out_tokens + (int64_t)b * (p.gamma + 1);
    for (int i = lane; i <= p.gamma; i += 64)
        out[i] = i < n ? drafted : (i == n ? s_t[n] : -1);       // (i < n implies i = lane < gamma)
    if (lane == 0) p.n_accepted[b] = n;
}

// -------------------------------------------------------------- sampling ----
// rows 0..gamma: target rows; rows gamma+1..2*gamma: draft rows 0..gamma-1
__global__ __launch_bounds__(256)
void accept_softmax_partial(const AcceptParams p)
{
    __shared__ float s_m[4], s_z[4];
    const int chunk = blockIdx.x, row = blockIdx.y, b = blockIdx.z;
    const float* x = row <= p.gamma
        ? p.target + ((int64_t)b * (p.gamma + 1) + row) * p.vocab
        : p.draft + ((int64_t)b * p.gamma + (row - p.gamma - 1)) * p.vocab;
    const int lo = chunk * kAccChunk, hi = min(p.vocab, lo + kAccChunk);
    // the thread's whole share is requested up front and kept for the second pass
    float y[kAccPerThread];
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) {
        const int v = lo + j * 256 + threadIdx.x;
        y[j] = v < hi ? x[v] * p.inv_t_log2 : -INFINITY;
    }
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) m = fmaxf(m, y[j]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) s_m[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) z += fast_exp2(y[j] - m);       // (-inf padding adds 0)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) z += __shfl_xor(z, off);
    if (lane == 0) s_z[wave] = z;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int64_t slot = ((int64_t)b * (2 * p.gamma + 1) + row) * p.n_chunks + chunk;
        p.part_val[slot] = m;
        p.part_aux[slot] = (s_z[0] + s_z[1]) + (s_z[2] + s_z[3]);
    }
}

// Merged (max, sum exp) of every row from the pass-1 partials, into LDS.
__device__ __forceinline__ void accept_merge_rows(const AcceptParams& p, int b, int rows, float* s_m, float* s_z)
{
    for (int row = threadIdx.x; row < rows; row += blockDim.x) {
        const int64_t slot = ((int64_t)b * rows + row) * p.n_chunks;
        float m = -INFINITY, z = 0.f;
        for (int c0 = 0; c0 < p.n_chunks; c0 += 8) {         // eight chunks' loads in flight at a time
            float pm[8], pz[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = c0 + j < p.n_chunks;
                pm[j] = in ? p.part_val[slot + c0 + j] : -INFINITY;
                pz[j] = in ? p.part_aux[slot + c0 + j] : 0.f;
            }
            float mc = m;
#pragma unroll
            for (int j = 0; j < 8; ++j) mc = fmaxf(mc, pm[j]);
            z *= (mc == -INFINITY) ? 0.f : fast_exp2(m - mc);
#pragma unroll
            for (int j = 0; j < 8; ++j) z += (pz[j] > 0.f) ? pz[j] * fast_exp2(pm[j] - mc) : 0.f;
            m = mc;
        }
        s_m[row] = m; s_z[row] = z;
    }
}

// weight of token v at the first rejected position: residual max(p - q, 0), or p when nothing was rejected
struct AcceptWeight {
    const float* trow;
    const float* drow;        // null: no residual
    float inv_t_log2, mt, inv_zt, md, inv_zd;
    __device__ __forceinline__ float operator()(int v) const
    {
        const float pv = fast_exp2(trow[v] * inv_t_log2 - mt) * inv_zt;
        if (!drow) return pv;
        const float qv = fast_exp2(drow[v] * inv_t_log2 - md) * inv_zd;
        return fmaxf(pv - qv, 0.f);
    }
};

__device__ __forceinline__ AcceptWeight accept_weight(const AcceptParams& p, int b, int n, float mt, float zt, float md, float zd)
{
    AcceptWeight w;
    const bool residual = n < p.gamma;
    w.trow = p.target + ((int64_t)b * (p.gamma + 1) + n) * p.vocab;
    w.drow = residual ? p.draft + ((int64_t)b * p.gamma + n) * p.vocab : nullptr;
    w.inv_t_log2 = p.inv_t_log2;
    w.mt = mt; w.inv_zt = 1.f / zt;
    w.md = residual ? md : 0.f; w.inv_zd = residual ? 1.f / zd : 0.f;
    return w;
}

__global__ __launch_bounds__(256)
void accept_mass_partial(const AcceptParams p)
{
    __shared__ float s_m[129], s_z[129];        // merged (max, sum) of up to 2*gamma+1 rows
    __shared__ float s_part[4];
    __shared__ int s_n;
    const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rows = 2 * p.gamma + 1;
    accept_merge_rows(p, b, rows, s_m, s_z);
    __syncthreads();
    // The gamma accept tests, one per lane of the first wave (gamma <= 64): every test's loads
    // are in flight together; the first failing test is found by a ballot.
    if (wave == 0) {
        const float* tgt = p.target + (int64_t)b * (p.gamma + 1) * p.vocab;
        const float* drf = p.draft + (int64_t)b * p.gamma * p.vocab;
        bool ok = true;
        if (lane < p.gamma) {
            const int tok = p.tokens[(int64_t)b * p.gamma + lane];
            ok = tok >= 0 && tok < p.vocab;                      // not a token: cannot be accepted
            if (ok) {
                const float pt = fast_exp2(tgt[(int64_t)lane * p.vocab + tok] * p.inv_t_log2 - s_m[lane]) / s_z[lane];
                const float qd = fast_exp2(drf[(int64_t)lane * p.vocab + tok] * p.inv_t_log2 - s_m[p.gamma + 1 + lane]) /
                                 s_z[p.gamma + 1 + lane];
                ok = p.uniforms[(int64_t)b * (p.gamma + 1) + lane] * qd < pt;
            }
        }
        const uint64_t failed = __ballot(!ok);
        if (lane == 0) s_n = failed ? __ffsll((long long)failed) - 1 : p.gamma;
    }
    __syncthreads();
    const int n = s_n;
    if (chunk == 0) {                                            // what pass 3 needs of the above
        if (tid < rows) { p.norm[((int64_t)b * rows + tid) * 2] = s_m[tid]; p.norm[((int64_t)b * rows + tid) * 2 + 1] = s_z[tid]; }
        if (tid == 0) p.n_rej[b] = n;
    }
    const int dn = n < p.gamma ? p.gamma + 1 + n : 0;
    const AcceptWeight weight = accept_weight(p, b, n, s_m[n], s_z[n], s_m[dn], s_z[dn]);
    const int lo = chunk * kAccChunk, hi = min(p.vocab, lo + kAccChunk);
    float w[kAccPerThread];
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) {
        const int v = lo + j * 256 + tid;
        w[j] = v < hi ? weight(v) : 0.f;
    }
    float mine = 0.f;
#pragma unroll
    for (int j = 0; j < kAccPerThread; ++j) mine += w[j];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mine += __shfl_xor(mine, off);
    if (lane == 0) s_part[wave] = mine;
    __syncthreads();
    if (tid == 0) p.chunk_mass[(int64_t)b * p.n_chunks + chunk] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

__global__ __launch_bounds__(kAccThreads)
void accept_sample_final(const AcceptParams p)
{
    __shared__ float s_w[kAccWaves];
    __shared__ int s_idx[kAccWaves];
    __shared__ int s_y;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rows = 2 * p.gamma + 1;
    const int n = p.n_rej[b];
    const int dn = n < p.gamma ? p.gamma + 1 + n : 0;
    const float* nm = p.norm + (int64_t)b * rows * 2;
    const AcceptWeight weight = accept_weight(p, b, n, nm[2 * n], nm[2 * n + 1], nm[2 * dn], nm[2 * dn + 1]);
    const float* cm = p.chunk_mass + (int64_t)b * p.n_chunks;
    if (tid == 0) s_y = -1;
    // total mass and the owner of the goal among the chunks: the LAST chunk with mass whose prefix
    // does not exceed the goal -- exactly one chunk, whatever rounding did to the sums (a goal that
    // rounding put at or beyond the total lands on the last chunk with mass).  Every thread walks
    // the same few numbers in the same order.
    float W = 0.f;
    for (int c = 0; c < p.n_chunks; ++c) W += cm[c];
    if (!(W > 0.f)) {
        // no residual mass (p == q): fall back to the target's most likely token
        const int seg = ((p.vocab + kAccWaves - 1) / kAccWaves + 63) & ~63;
        const int lo = min(p.vocab, wave * seg), hi = min(p.vocab, lo + seg);
        float bv = 0.f; int bi = -1;
        for (int v = lo + lane; v < hi; v += 64) {
            const float y = weight.trow[v];
            if (bi < 0 || y > bv) { bv = y; bi = v; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oi = __shfl_xor(bi, off);
            argmax_merge(bv, bi, ov, oi);
        }
        if (lane == 0) { s_w[wave] = bv; s_idx[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kAccWaves; ++w) argmax_merge(bv, bi, s_w[w], s_idx[w]);
            s_y = bi;
        }
        __syncthreads();
    } else {
        const float goal = p.uniforms[(int64_t)b * (p.gamma + 1) + p.gamma] * W;
        int own1 = -1;
        float pre1 = 0.f, acc1 = 0.f;
        for (int c = 0; c < p.n_chunks; ++c) {
            const float m = cm[c];
            if (m > 0.f && acc1 <= goal) { own1 = c; pre1 = acc1; }
            acc1 += m;
        }
        // Inside the owning chunk the same rule picks a wave's share (the chunk is dealt to the
        // waves in token order), and the owning wave walks its few hundred tokens 64 at a time for
        // the first token whose cumulative mass passes the goal, else takes its last token with mass.
        const int lo1 = own1 * kAccChunk, hi1 = min(p.vocab, lo1 + kAccChunk);
        const int seg2 = ((hi1 - lo1 + kAccWaves - 1) / kAccWaves + 63) & ~63;
        const int lo2 = min(hi1, lo1 + wave * seg2), hi2 = min(hi1, lo2 + seg2);
        float mine2 = 0.f;
#pragma unroll 8
        for (int v = lo2 + lane; v < hi2; v += 64) mine2 += weight(v);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mine2 += __shfl_xor(mine2, off);
        if (lane == 0) s_w[wave] = mine2;
        __syncthreads();
        int own2 = -1;
        float pre2 = pre1, acc2 = pre1;
#pragma unroll
        for (int w = 0; w < kAccWaves; ++w) {
            if (s_w[w] > 0.f && acc2 <= goal) { own2 = w; pre2 = acc2; }
            acc2 += s_w[w];
        }
        // (rounding can leave the chunk's own waves without mass although the chunk had some: the
        // first wave then reports the chunk's last token with mass, or its first token)
        if (own2 < 0) own2 = 0;
        if (wave == own2) {
            float c = pre2;
            int y = -1, last = -1;
            for (int base = lo2; base < hi2; base += 64) {       // (at most eight steps)
                const int v = base + lane;
                const float w = v < hi2 ? weight(v) : 0.f;
                float incl = w;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const float t = __shfl_up(incl, off);
                    if (lane >= off) incl += t;
                }
                const uint64_t massive = __ballot(w > 0.f);
                const uint64_t passed = __ballot(w > 0.f && c + incl > goal);
                if (massive) last = base + 63 - __builtin_clzll(massive);
                if (passed && y < 0) y = base + __ffsll((long long)passed) - 1;
                c += __shfl(incl, 63);
            }
            if (lane == 0) s_y = y >= 0 ? y : (last >= 0 ? last : lo1);
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int32_t* x = p.tokens + (int64_t)b * p.gamma;
        int32_t* out = p.out_tokens + (int64_t)b * (p.gamma + 1);
        for (int i = 0; i <= p.gamma; ++i) out[i] = i < n ? x[i] : (i == n ? s_y : -1);
        p.n_accepted[b] = n;
    }
}

// ------------------------------------------------------------------ tree ----
// Greedy walk over a static draft tree (App. B): rows of target_logits are tree
// nodes; node 0 is the last committed token, parent[i] < i.  One wave per
// request: lane i merges the per-chunk argmax partials of node i and holds its
// parent and drafted token; the wave walks from the root, moving to the
// lowest-numbered child that drafted the target's token (found by a ballot).
__global__ __launch_bounds__(64)
void accept_tree_final(const AcceptParams p, const int32_t* parent, int32_t* accepted_nodes)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int n_nodes = p.gamma + 1;                             // <= 64: lane i holds node i
    __shared__ int s_t[64];
    const int32_t* x = p.tokens + (int64_t)b * n_nodes;
    const int my_tok = lane < n_nodes ? x[lane] : -1;            // (in flight while the partials are merged)
    const int my_par = lane < n_nodes ? parent[lane] : -1;       // parent[] is shared by the batch
    if (lane < n_nodes) {
        float bv = 0.f; int bi = -1;
        const int64_t slot = ((int64_t)b * n_nodes + lane) * p.n_chunks;
        for (int c0 = 0; c0 < p.n_chunks; c0 += 8) {             // eight chunks' loads in flight at a time
            float pv[8]; int pi[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = c0 + j < p.n_chunks;
                pv[j] = in ? p.part_val[slot + c0 + j] : 0.f;
                pi[j] = in ? __float_as_int(p.part_aux[slot + c0 + j]) : -1;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) argmax_merge(bv, bi, pv[j], pi[j]);
        }
        s_t[lane] = bi;
    }
    __syncthreads();
    int32_t* out = p.out_tokens + (int64_t)b * n_nodes;
    int32_t* nodes = accepted_nodes + (int64_t)b * n_nodes;
    // the walk: every lane follows it; the children of the current node that drafted the target's
    // token answer a ballot, the lowest-numbered one is taken (at most n_nodes - 1 steps)
    int cur = 0, n = 0;
    int my_out = -1, my_node = -1;                               // lane i ends up holding out[i] and nodes[i]
    for (;;) {
        const int t = s_t[cur];
        const uint64_t match = __ballot(lane > cur && lane < n_nodes && my_par == cur && my_tok == t);
        if (!match) { if (lane == n) my_out = t; break; }
        const int next = __ffsll((long long)match) - 1;
        const int tok_next = __shfl(my_tok, next);
        if (lane == n) { my_node = next; my_out = tok_next; }
        ++n; cur = next;
    }
    if (lane < n_nodes) { out[lane] = my_out; nodes[lane] = my_node; }
    if (lane == 0) p.n_accepted[b] = n;
}

static int accept_chunks(int vocab) { return (vocab + kAccChunk - 1) / kAccChunk; }

}  // namespace specvlm

using namespace specvlm;

extern "C" size_t specvlm_accept_workspace_bytes(int batch, int gamma, int vocab, int sampling)
{
    if (batch <= 0 || gamma < 0 || vocab < 1) return 0;
    const size_t rows = sampling ? 2 * (size_t)gamma + 1 : (size_t)gamma + 1;
    size_t bytes = 2 * align256((size_t)batch * rows * accept_chunks(vocab) * sizeof(float));
    if (sampling)       // merged row statistics, chunk masses of the rejected row, rejected positions
        bytes += align256((size_t)batch * rows * 2 * sizeof(float)) +
                 align256((size_t)batch * accept_chunks(vocab) * sizeof(float)) +
                 align256((size_t)batch * sizeof(int32_t));
    return bytes;
}

extern "C" int specvlm_accept(
    const float* target_logits, const float* draft_logits,
    const int32_t* draft_tokens, const float* uniforms,
    int batch, int gamma, int vocab, float temperature,
    int32_t* n_accepted, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch < 0 || gamma < 0 || vocab < 1) return SPECVLM_EINVAL;
    const bool sampling = uniforms != nullptr;
    if (!sampling && draft_logits) return SPECVLM_EINVAL;            // draft logits without uniforms
    if (sampling && gamma > 0 && !draft_logits) return SPECVLM_EINVAL;
    if (sampling && !(temperature > 0.f && temperature < INFINITY)) return SPECVLM_EINVAL;
    if (gamma > 64) return SPECVLM_EUNSUPPORTED;
    if (batch == 0) return SPECVLM_OK;
    if (!target_logits || !n_accepted || !out_tokens || (gamma > 0 && !draft_tokens)) return SPECVLM_EINVAL;
    if (batch > 65535) return SPECVLM_EUNSUPPORTED;
    const size_t need = specvlm_accept_workspace_bytes(batch, gamma, vocab, sampling);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SPECVLM_EWORKSPACE;

    AcceptParams p;
    p.target = target_logits; p.draft = draft_logits; p.tokens = draft_tokens; p.uniforms = uniforms;
    p.batch = batch; p.gamma = gamma; p.vocab = vocab; p.n_chunks = accept_chunks(vocab);
    p.inv_t_log2 = sampling ? kLog2e / temperature : kLog2e;
    p.n_accepted = n_accepted; p.out_tokens = out_tokens;
    const size_t rows = sampling ? 2 * (size_t)gamma + 1 : (size_t)gamma + 1;
    const size_t part_bytes = align256((size_t)batch * rows * p.n_chunks * sizeof(float));
    char* ws = (char*)workspace;
    p.part_val = (float*)ws;
    p.part_aux = (float*)(ws + part_bytes);
    p.norm = (float*)(ws + 2 * part_bytes);
    p.chunk_mass = (float*)((char*)p.norm + align256((size_t)batch * rows * 2 * sizeof(float)));
    p.n_rej = (int32_t*)((char*)p.chunk_mass + align256((size_t)batch * p.n_chunks * sizeof(float)));
    hipStream_t s = (hipStream_t)stream;
    if (!sampling) {
        hipLaunchKernelGGL(accept_argmax_partial, dim3(p.n_chunks, gamma + 1, batch), dim3(256), 0, s, p);
        hipLaunchKernelGGL(accept_greedy_final, dim3(batch), dim3(64), 0, s, p);
    } else {
        hipLaunchKernelGGL(accept_softmax_partial, dim3(p.n_chunks, 2 * gamma + 1, batch), dim3(256), 0, s, p);
        hipLaunchKernelGGL(accept_mass_partial, dim3(p.n_chunks, batch), dim3(256), 0, s, p);
        hipLaunchKernelGGL(accept_sample_final, dim3(batch), dim3(kAccThreads), 0, s, p);
    }
    return launch_status();
}

extern "C" size_t specvlm_accept_tree_workspace_bytes(int batch, int n_nodes, int vocab)
{
    return specvlm_accept_workspace_bytes(batch, n_nodes - 1, vocab, 0);
}

extern "C" int specvlm_accept_tree(
    const float* target_logits, const int32_t* node_tokens, const int32_t* parent,
    int batch, int n_nodes, int vocab,
    int32_t* n_accepted, int32_t* accepted_nodes, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch < 0 || n_nodes < 1 || vocab < 1) return SPECVLM_EINVAL;
    if (n_nodes > 64) return SPECVLM_EUNSUPPORTED;
    if (batch == 0) return SPECVLM_OK;
    if (!target_logits || !node_tokens || !parent || !n_accepted || !accepted_nodes || !out_tokens)
        return SPECVLM_EINVAL;
    if (batch > 65535) return SPECVLM_EUNSUPPORTED;
    const size_t need = specvlm_accept_tree_workspace_bytes(batch, n_nodes, vocab);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SPECVLM_EWORKSPACE;
    AcceptParams p;
    p.target = target_logits; p.draft = nullptr; p.tokens = node_tokens; p.uniforms = nullptr;
    p.batch = batch; p.gamma = n_nodes - 1; p.vocab = vocab; p.n_chunks = accept_chunks(vocab);
    p.inv_t_log2 = kLog2e;
    p.n_accepted = n_accepted; p.out_tokens = out_tokens;
    p.part_val = (float*)workspace;
    p.part_aux = (float*)((char*)workspace + need / 2);
    p.norm = nullptr; p.chunk_mass = nullptr; p.n_rej = nullptr;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(accept_argmax_partial, dim3(p.n_chunks, n_nodes, batch), dim3(256), 0, s, p);
    hipLaunchKernelGGL(accept_tree_final, dim3(batch), dim3(64), 0, s, p, parent, accepted_nodes);
    return launch_status();
}
