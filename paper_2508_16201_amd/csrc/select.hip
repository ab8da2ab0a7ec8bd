// specvlm_select: the two-stage retention set of Sec. 3.2.
//   Stage I  : V_R = the k highest-scoring video tokens (ties -> lower index),
//              by a most-significant-digit radix select on order-preserving
//              integer keys (4 passes of 8 bits, wave-ballot aggregated
//              histograms in LDS).
//   Stage II : V_U = tokens of V \ V_R at the fixed fractional interval
//              I = R/U in raster order: remainder ranks floor(t*R/U), exact
//              integer arithmetic (Eq. 7 with the budget as denominator).
//   Output   : sort(V_R u V_U) by a stable compaction.
// One workgroup of 1024 threads per request; thread t owns the contiguous run
// of tokens [t*per, (t+1)*per) and keeps their keys in registers, so every
// "how many before me" question is one block-wide exclusive scan of popcounts.
#include <atomic>

#include "common.h"

namespace specvlm {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelCopies = 64;            // copies of the digit histogram in LDS (summed after every pass)
constexpr int kSelCopyWords = 257;        // a copy is 257 words long: the copies of one digit lie in different banks
constexpr size_t kSelHistBytes = 2ull * kSelCopies * kSelCopyWords * sizeof(int);   // two sets: the passes alternate

struct SelectParams {
    const float* scores;
    const int32_t* cu_video;
    const int32_t* k_top;
    const int32_t* keep_budget;
    const int32_t* cu_keep;
    int max_n_video;
    int32_t* keep_idx;
    uint8_t* from_topk;
    int32_t* status;
};

// Order-preserving key: larger score <=> larger key.  -0.0 is +0.0; NaN is the
// smallest key of all.
__device__ __forceinline__ uint32_t score_key(float x)
{
    if (x != x) return 0u;
    uint32_t u = __float_as_uint(x);
    if (x == 0.f) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// A thread's run of scores [first, first + per) of a request of n scores, four at a time (dword-aligned
// 16-byte loads); slots past the run or past n read as 0.  With one score per load every instruction
// would touch 64 different cache lines, and the address path takes a cycle per line: 13 such loads per
// thread were the longest phase of the select kernel.
template <int E>
__device__ __forceinline__ void load_run(const float* sc, int first, int per, int n, float (&raw)[E])
{
    typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
    for (int e4 = 0; e4 < E; e4 += 4) {
        const int idx = first + e4;
        if (e4 + 3 < per && idx + 3 < n) {
            const float4u v = *reinterpret_cast<const float4u*>(sc + idx);
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[e4 + i] = v[i];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[e4 + i] = (e4 + i < per && idx + i < n) ? sc[idx + i] : 0.f;
        }
    }
}

// Exclusive prefix sums of two ints per thread in one round of barriers.
__device__ __forceinline__ void block_excl_scan2(int a, int b, int (*s_wave2)[kSelWaves], int* a_before, int* b_before)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ia = a, ib = b;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int ya = __shfl_up(ia, off), yb = __shfl_up(ib, off);
        if (lane >= off) { ia += ya; ib += yb; }
    }
    if (lane == 63) { s_wave2[0][wave] = ia; s_wave2[1][wave] = ib; }
    __syncthreads();
    int wa = 0, wb = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        if (w < wave) { wa += s_wave2[0][w]; wb += s_wave2[1][w]; }
    }
    *a_before = wa + ia - a;
    *b_before = wb + ib - b;
}

template <int E>
__global__ __launch_bounds__(kSelThreads)
void select_kernel(const SelectParams p)
{
    // kSelCopies copies of the digit histogram (padded: see below); the passes alternate between two sets
    extern __shared__ int s_hist_dyn[];
    int (*s_hist)[kSelCopies][kSelCopyWords] = reinterpret_cast<int (*)[kSelCopies][kSelCopyWords]>(s_hist_dyn);
    __shared__ int s_part[4][256];
    __shared__ int s_wave2[2][kSelWaves];
    __shared__ int s_pick[3];

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v0 = p.cu_video ? p.cu_video[b] : 0;
    const int n = p.cu_video ? p.cu_video[b + 1] - v0 : p.max_n_video;
    // The scores are requested first (guarded by the token count alone, so always in bounds); the
    // request's sizes, one more memory round trip away, are fetched while those loads are in flight.
    const int per = n > 0 ? (n + kSelThreads - 1) / kSelThreads : 0;
    const int first = tid * per;
    const float* sc = p.scores + v0;
    float raw[E];
    load_run<E>(sc, first, per, n, raw);
    // the first pass's histograms are cleared while the scores are on their way
    for (int i = tid; i < kSelCopies * kSelCopyWords; i += kSelThreads) (&s_hist[0][0][0])[i] = 0;
    const int k = p.k_top[b], budget = p.keep_budget[b];
    const int out0 = p.cu_keep ? p.cu_keep[b] : 0;
    const bool bad = n < 0 || n > E * kSelThreads || n > p.max_n_video || k < 0 || k > budget || budget > n;
    if (p.status && tid == 0) p.status[b] = bad ? SPECVLM_EINVAL : SPECVLM_OK;
    if (bad || budget == 0) return;

    uint32_t key[E];
    uint64_t valid = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int idx = first + e;
        const bool ok = e < per && idx < n;                     // (per <= E once the sizes are valid)
        key[e] = ok ? score_key(raw[e]) : 0u;
        if (ok) valid |= 1ull << e;
    }

    // ---- Stage I: radix select of the k-th largest key ----
    uint32_t prefix = 0, known = 0;
    int need = k;                       // how many still to take inside the current prefix
    if (k > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (pass == 0) __syncthreads();             // the cleared histograms are visible
            // The copies are summed afterwards, so a lane may add to any of them: every lane of an
            // instruction has a copy of its own (an LDS atomic serialises over the lanes that hit one
            // address, and the leading digit of attention scores, sign and exponent, takes only a handful
            // of values), the waves start at different copies, and a copy is 257 words long, so the copies
            // of a digit lie in different banks.  No aggregation over the wave or over a thread's keys:
            // both were measured and cost more than the additions they save.
            int* const my_hist = &s_hist[pass & 1][(4 * wave + lane) & (kSelCopies - 1)][0];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const bool match = ((valid >> e) & 1) && ((key[e] & known) == prefix);
                if (match) atomicAdd(&my_hist[(key[e] >> shift) & 255], 1);
            }
            // the other set (read for the last time two barriers ago) is cleared for the next pass
            if (pass < 3)
                for (int i = tid; i < kSelCopies * kSelCopyWords; i += kSelThreads) (&s_hist[(pass + 1) & 1][0][0])[i] = 0;
            __syncthreads();
            {
                // thread (quarter, digit) sums a quarter of the digit's copies; the four quarters sit in
                // the lanes of four different waves, so they meet in LDS
                const int digit = tid & 255, quarter = tid >> 8;
                int t = 0;
#pragma unroll
                for (int w = 0; w < kSelCopies / 4; ++w) t += s_hist[pass & 1][quarter * (kSelCopies / 4) + w][digit];
                s_part[quarter][digit] = t;
            }
            __syncthreads();
            if (wave == 0) {
                // lane l owns digits 4l..4l+3; suffix sums from the top digit down
                int c4[4], mine = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    c4[i] = s_part[0][4 * lane + i] + s_part[1][4 * lane + i] + s_part[2][4 * lane + i] + s_part[3][4 * lane + i];
                    mine += c4[i];
                }
                int incl = mine;                        // inclusive suffix sum over lanes >= lane
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int y = __shfl_down(incl, off);
                    if (lane + off < 64) incl += y;
                }
                int above = incl - mine;                // keys in digits owned by higher lanes
                if (above < need && need <= incl) {
#pragma unroll
                    for (int i = 3; i >= 0; --i) {
                        if (above < need && need <= above + c4[i]) {
                            s_pick[0] = 4 * lane + i;
                            s_pick[1] = need - above;
                            s_pick[2] = (need - above == c4[i]);    // the whole bucket is taken: nothing left to rank
                        }
                        above += c4[i];
                    }
                }
            }
            __syncthreads();
            prefix |= (uint32_t)s_pick[0] << shift;
            known |= 255u << shift;
            need = s_pick[1];
            // When the keys that share the digits known so far are exactly as many as are still needed,
            // all of them are taken and the lower digits decide nothing: the remaining passes are skipped
            // (with distinct scores this is the usual case after three passes).
            if (s_pick[2]) break;
        }
    }
    // now: prefix = the known digits of the k-th largest key (all four, or fewer when a whole bucket
    // is taken); take every key above it and the first `need` keys that share it, in index order.
    uint64_t gt = 0, eq = 0;
    if (k > 0) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (!((valid >> e) & 1)) continue;
            const uint32_t kk = key[e] & known;
            if (kk > prefix) gt |= 1ull << e;
            else if (kk == prefix) eq |= 1ull << e;
        }
    }
    // One block scan gives every thread the numbers of larger and of equal keys before its
    // tokens; everything else that is "before me" follows in closed form: the tokens before mine
    // are min(first, n), those taken by Stage I are the larger ones plus the equal ones up to
    // `need`, the rest is my first remainder rank, and the stride picks below that rank are counted
    // by the stride formula itself.
    int gt_before, eq_before;
    block_excl_scan2(__popcll(gt), __popcll(eq), s_wave2, &gt_before, &eq_before);
    int take = need - eq_before;
    take = take < 0 ? 0 : take;
    const int top_before = gt_before + (eq_before < need ? eq_before : need);
    uint64_t top = gt;
    for (uint64_t m = eq; m && take > 0; --take) {
        const uint64_t bit = m & (~m + 1);
        top |= bit;
        m ^= bit;
    }

    // ---- Stage II: uniform stride over the remainder ----
    const uint64_t rem_mask = valid & ~top;
    const int rho_before = (first < n ? first : n) - top_before;
    // n <= 65536, so every product below (rank x U, index x R, each factor <= 65536 and one of them
    // < 65536) fits 32 bits: unsigned 32-bit divisions, exact
    const uint32_t R = (uint32_t)(n - k), U = (uint32_t)(budget - k);
    uint64_t uni = 0;
    int uni_before = 0;                                           // stride picks with a rank below mine
    if (U > 0) {
        uint32_t t = (uint32_t)(((uint64_t)rho_before * U + R - 1) / R);   // first stride index at or after my ranks
        uni_before = (int)(t < U ? t : U);
        if (t < U && rem_mask) {
            const uint32_t tr = t * R;                            // t <= U - 1: the product fits
            uint32_t q = tr / U, frac = tr % U;                   // rank floor(t*R/U)
            const uint32_t step_q = R / U, step_f = R % U;
            uint32_t rho = (uint32_t)rho_before;
            for (uint64_t m = rem_mask; m && t < U; ++rho) {
                const uint64_t bit = m & (~m + 1);
                m ^= bit;
                if (rho == q) {
                    uni |= bit;
                    ++t; q += step_q; frac += step_f;
                    if (frac >= U) { frac -= U; ++q; }
                }
            }
        }
    }

    // ---- stable compaction of V_R u V_U: my first output position is what was kept before me ----
    const uint64_t keep = top | uni;
    int pos = out0 + top_before + uni_before;
    for (uint64_t m = keep; m;) {
        const int e = __ffsll((long long)m) - 1;
        m &= m - 1;
        p.keep_idx[pos] = first + e;
        if (p.from_topk) p.from_topk[pos] = (uint8_t)((top >> e) & 1);
        ++pos;
    }
}


// ---------------------------------------------------------------------------
// Stage I's own size rule (Sec. 3.2, Eq. 6): the smallest c such that the c
// largest scores reach lambda of the total score mass.  Same radix descent as
// the selection, but the per-digit histograms carry the MASS of the keys, not
// their number (the first pass's sums also give the total); the numbers of keys
// above and at the threshold are counted once, at the end.
// Sums are 64-bit fixed point (score * 2^40 / max score): integer adds commute,
// so the result does not depend on the order in which lanes reach the atomics.
// Scores are attention masses: a value that is not a finite positive number
// counts as 0 (and keeps its place in the descending order).
struct TopPParams {
    const float* scores;
    const int32_t* cu_video;
    int max_n_video;
    float lambda;
    const int32_t* max_count;
    int32_t* count;
};

constexpr size_t kTopPHistBytes = (size_t)kSelCopies * kSelCopyWords * sizeof(unsigned long long);   // one set

template <int E>
__global__ __launch_bounds__(kSelThreads)
void top_p_kernel(const TopPParams p)
{
    // 64 copies of the 256 per-digit mass sums, one copy per lane of an instruction as in the selection
    // (dynamic LDS); counts are not kept per digit: only the threshold key's are needed, at the end
    extern __shared__ unsigned long long s_mass_dyn[];
    unsigned long long (*s_mass)[kSelCopyWords] = reinterpret_cast<unsigned long long (*)[kSelCopyWords]>(s_mass_dyn);
    __shared__ unsigned long long s_part[4][256];
    __shared__ float s_redf[kSelWaves];
    __shared__ int s_redc[2][kSelWaves];
    __shared__ unsigned long long s_pick_sum, s_goal;
    __shared__ int s_pick;

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v0 = p.cu_video ? p.cu_video[b] : 0;
    const int n = p.cu_video ? p.cu_video[b + 1] - v0 : p.max_n_video;
    if (n <= 0 || n > E * kSelThreads) { if (tid == 0) p.count[b] = 0; return; }
    const int per = (n + kSelThreads - 1) / kSelThreads;
    const int first = tid * per;
    const float* sc = p.scores + v0;

    // a value that is not a finite positive number carries no mass; its key still ranks it
    auto mass_of = [](float x) { return (x > 0.f && x < INFINITY) ? x : 0.f; };
    float val[E];
    load_run<E>(sc, first, per, n, val);
    // the sums are cleared while the scores are on their way
    for (int i = tid; i < kSelCopies * kSelCopyWords; i += kSelThreads) (&s_mass[0][0])[i] = 0ull;
    uint64_t valid = 0;
    float mx = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int idx = first + e;
        const bool ok = e < per && idx < n;
        if (ok) valid |= 1ull << e;
        mx = fmaxf(mx, mass_of(val[e]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) s_redf[wave] = mx;
    __syncthreads();                                    // (also: the cleared sums are visible)
    mx = 0.f;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) mx = fmaxf(mx, s_redf[w]);
    if (!(mx > 0.f)) { if (tid == 0) p.count[b] = 0; return; }

    // fixed point by an exact power-of-two scaling: the largest score lands in [2^39, 2^40)
    int mx_exp;
    (void)frexpf(mx, &mx_exp);
    const int fix_shift = 40 - mx_exp;
    auto to_fix = [&](float x) { return (unsigned long long)ldexpf(mass_of(x), fix_shift); };

    uint32_t prefix = 0, known = 0;
    unsigned long long above_sum = 0;          // mass of the keys known to rank above the threshold
    unsigned long long goal = 0;               // ceil(lambda * total), known once the first pass has the total
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        unsigned long long* const my_mass = &s_mass[(4 * wave + lane) & (kSelCopies - 1)][0];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float x = val[e];
            __asm__ volatile("" : "+v"(x));          // recompute key and mass per pass: keeps them out of registers
            const uint32_t key = score_key(x);
            if (((valid >> e) & 1) && ((key & known) == prefix)) {
                const unsigned long long m = to_fix(x);
                if (m) atomicAdd(&my_mass[(key >> shift) & 255], m);
            }
        }
        __syncthreads();
        {
            // thread (quarter, digit) sums a quarter of the digit's copies
            const int digit = tid & 255, quarter = tid >> 8;
            unsigned long long t = 0;
#pragma unroll
            for (int w = 0; w < kSelCopies / 4; ++w) t += s_mass[quarter * (kSelCopies / 4) + w][digit];
            s_part[quarter][digit] = t;
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l..4l+3; inclusive suffix sums from the top digit down
            unsigned long long m4[4], mmine = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                m4[i] = s_part[0][4 * lane + i] + s_part[1][4 * lane + i] + s_part[2][4 * lane + i] + s_part[3][4 * lane + i];
                mmine += m4[i];
            }
            unsigned long long mincl = mmine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned long long ym = __shfl_down(mincl, off);
                if (lane + off < 64) mincl += ym;
            }
            if (pass == 0) {
                // the first pass sees every key: lane 0's suffix sum is the total mass.
                // goal = ceil(lambda * total); lambda is an fp32 in [0,1] and total < 2^56, so the double
                // product is within a few units of 2^-40 of the largest score: far below the parity margin
                const unsigned long long total = __shfl(mincl, 0);
                const double goal_d = ceil((double)p.lambda * (double)total);
                goal = goal_d <= 0.0 ? 0ull : (unsigned long long)goal_d;
                if (goal > total) goal = total;
                if (lane == 0) s_goal = goal;
            }
            // the threshold digit: first digit from the top where the running mass reaches the goal
            unsigned long long m_above = above_sum + (mincl - mmine);
            if (goal > 0 && m_above < goal && goal <= above_sum + mincl) {
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                    if (m_above < goal && goal <= m_above + m4[i]) { s_pick = 4 * lane + i; s_pick_sum = m_above; }
                    m_above += m4[i];
                }
            }
        } else if (pass < 3) {
            // (the sums were read for the last time before the barrier above: cleared for the next pass)
            for (int i = tid - kWave; i < kSelCopies * kSelCopyWords; i += kSelThreads - kWave) (&s_mass[0][0])[i] = 0ull;
        }
        __syncthreads();
        if (pass == 0) {
            goal = s_goal;
            if (goal == 0) { if (tid == 0) p.count[b] = 0; return; }
        }
        prefix |= (uint32_t)s_pick << shift;
        known |= 255u << shift;
        above_sum = s_pick_sum;
    }
    // prefix is now the threshold key: count the keys above it and those equal to it
    int gt = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const uint32_t key = score_key(val[e]);
        if ((valid >> e) & 1) { gt += key > prefix; eq += key == prefix; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { gt += __shfl_xor(gt, off); eq += __shfl_xor(eq, off); }
    if (lane == 0) { s_redc[0][wave] = gt; s_redc[1][wave] = eq; }
    __syncthreads();
    if (tid == 0) {
        int above_cnt = 0, eq_cnt = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) { above_cnt += s_redc[0][w]; eq_cnt += s_redc[1][w]; }
        // every key equal to the threshold carries the same mass: take as many as the goal needs
        const uint32_t u = (prefix & 0x80000000u) ? (prefix & 0x7fffffffu) : ~prefix;
        const float tval = __uint_as_float(u);
        const unsigned long long each = to_fix(tval);
        const unsigned long long need = goal - above_sum;
        long long take = each > 0 ? (long long)((need + each - 1) / each) : eq_cnt;
        if (take > eq_cnt) take = eq_cnt;
        if (take < 1) take = 1;
        int c = above_cnt + (int)take;
        if (p.max_count && c > p.max_count[b]) c = p.max_count[b];
        p.count[b] = c;
    }
}

// The histogram copies take more LDS than a kernel gets by default: the limit is raised once per
// device (the attribute belongs to the kernel as loaded on one device).
template <int E>
static int launch_select(int batch, const SelectParams& p, hipStream_t stream)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> raised[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECVLM_ELAUNCH;
    if (!raised[dev].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<E>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelHistBytes) != hipSuccess)
            return SPECVLM_ELAUNCH;
        raised[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(select_kernel<E>, dim3(batch), dim3(kSelThreads), kSelHistBytes, stream, p);
    return SPECVLM_OK;
}

template <int E>
static int launch_top_p(int batch, const TopPParams& p, hipStream_t stream)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> raised[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECVLM_ELAUNCH;
    if (!raised[dev].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&top_p_kernel<E>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kTopPHistBytes) != hipSuccess)
            return SPECVLM_ELAUNCH;
        raised[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(top_p_kernel<E>, dim3(batch), dim3(kSelThreads), kTopPHistBytes, stream, p);
    return SPECVLM_OK;
}

}  // namespace specvlm

using namespace specvlm;

extern "C" size_t specvlm_select_workspace_bytes(int batch, int max_n_video)
{
    (void)batch; (void)max_n_video;
    return 0;                           // everything lives in registers and LDS
}

extern "C" int specvlm_select(
    const float* scores, const int32_t* cu_video,
    const int32_t* k_top, const int32_t* keep_budget, const int32_t* cu_keep,
    int batch, int max_n_video, int total_keep,
    int32_t* keep_idx, uint8_t* from_topk, int32_t* status,
    void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    if (batch < 0 || max_n_video < 0 || total_keep < 0) return SPECVLM_EINVAL;
    if (batch == 0) return SPECVLM_OK;
    if (!k_top || !keep_budget) return SPECVLM_EINVAL;
    if (batch > 1 && (!cu_video || !cu_keep)) return SPECVLM_EINVAL;
    if ((int64_t)total_keep > (int64_t)batch * max_n_video) return SPECVLM_EINVAL;
    if (max_n_video > 64 * kSelThreads) return SPECVLM_EUNSUPPORTED;
    if (max_n_video == 0 || total_keep == 0) {
        // nothing can be kept; still report per-request status
        if (!status) return SPECVLM_OK;
    }
    if (total_keep > 0 && (!scores || !keep_idx)) return SPECVLM_EINVAL;

    SelectParams p;
    p.scores = scores; p.cu_video = cu_video; p.k_top = k_top; p.keep_budget = keep_budget;
    p.cu_keep = cu_keep; p.max_n_video = max_n_video;
    p.keep_idx = keep_idx; p.from_topk = from_topk; p.status = status;
    hipStream_t s = (hipStream_t)stream;
    const int per = (max_n_video + kSelThreads - 1) / kSelThreads;
    int rc;
    if (per <= 4)       rc = launch_select<4>(batch, p, s);
    else if (per <= 16) rc = launch_select<16>(batch, p, s);
    else if (per <= 32) rc = launch_select<32>(batch, p, s);
    else                rc = launch_select<64>(batch, p, s);
    if (rc != SPECVLM_OK) return rc;
    return launch_status();
}

extern "C" size_t specvlm_top_p_count_workspace_bytes(int batch, int max_n_video)
{
    (void)batch; (void)max_n_video;
    return 0;
}

extern "C" int specvlm_top_p_count(
    const float* scores, const int32_t* cu_video, int batch, int max_n_video,
    float lambda, const int32_t* max_count, int32_t* count,
    void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    if (batch < 0 || max_n_video < 0) return SPECVLM_EINVAL;
    if (!(lambda >= 0.f && lambda <= 1.f)) return SPECVLM_EINVAL;
    if (batch == 0) return SPECVLM_OK;
    if (!count || (max_n_video > 0 && !scores)) return SPECVLM_EINVAL;
    if (batch > 1 && !cu_video) return SPECVLM_EINVAL;
    if (max_n_video > 64 * kSelThreads) return SPECVLM_EUNSUPPORTED;
    TopPParams p;
    p.scores = scores; p.cu_video = cu_video; p.max_n_video = max_n_video;
    p.lambda = lambda; p.max_count = max_count; p.count = count;
    hipStream_t s = (hipStream_t)stream;
    const int per = (max_n_video + kSelThreads - 1) / kSelThreads;
    int rc;
    if (per <= 4)       rc = launch_top_p<4>(batch, p, s);
    else if (per <= 16) rc = launch_top_p<16>(batch, p, s);
    else if (per <= 32) rc = launch_top_p<32>(batch, p, s);
    else                rc = launch_top_p<64>(batch, p, s);
    if (rc != SPECVLM_OK) return rc;
    return launch_status();
}
