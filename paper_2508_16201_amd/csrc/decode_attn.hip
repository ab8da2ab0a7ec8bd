// specvlm_decode_attn: grouped-query softmax attention of a short query block
// (1 query for plain decode, gamma+1 for parallel verification; Sec. 2.1 of the
// paper) over a long bf16 KV cache, in split-K (flash-decode) form for gfx950.
//
// Work decomposition
//   One workgroup owns one (request, kv head, key split).  All G*q_len query
//   rows that share the kv head are packed into MFMA row blocks of 16 (MB of
//   them, MB <= 4), so every K/V byte is read from HBM exactly once.  The
//   workgroup has MB*KS compute waves -- wave (mb, ks) owns row block mb and
//   every KS-th 32-key chunk of each tile, so a wave carries one 16-row
//   accumulator only -- and, in the multi-query shapes, two or four loader
//   waves that do nothing but issue the tile loads: a direct-to-LDS load of
//   1 KB holds its wave for about 70 cycles, eight of them per tile are a
//   quarter of a tile's time when the waves that compute have to issue them.
//   More than 64 rows per kv head are cut into row groups, one workgroup each.
//
// Data movement
//   K/V tiles of TK keys stream HBM -> LDS with direct-to-LDS loads
//   (global_load_lds_dwordx4: no registers in between) into a ring of NS
//   stages; NS-1 tiles are in flight while one is consumed.  A stage is
//   released by one s_barrier per tile, which all waves pass; before it the
//   loader waves wait on their own vmcnt for the tile about to be read, never
//   on the younger tiles.  K rows are
//   stored with their 16-byte chunks XOR-swizzled by the key index so that the
//   MFMA operand reads (16 keys x one chunk per 16 lanes) hit distinct banks;
//   the swizzle is applied on the global-address side, the LDS side of a
//   direct load being fixed (lane * 16 bytes).  The Q fragments take the same
//   road (HBM -> LDS -> registers): with no load returning into registers the
//   compiler has nothing to guard with a wait that would drain the ring, and
//   the waits the kernel places itself are the only ones in the sweep.  A cache
//   of 8 MB or more per launch is read with non-temporal loads.
//
// Placement
//   Workgroup ids run over the kv heads fastest; ids are dealt to the 8 XCDs
//   round-robin, so with 8 kv heads all splits of a head and the merge of that
//   head share one XCD and its L2, where the partials (bf16 outputs, fp32
//   maxima and sums) stay between the two kernels.  A single request is cut
//   into about 192 workgroups in one round (HBM saturates before every CU is
//   busy); ragged batches of up to 64 requests into balanced pieces (equal runs
//   of key tiles per group of workgroups, see below), larger ones into splits
//   of at most 2048 keys that the dispatcher can balance.
//
// MFMA formulation (v_mfma_f32_16x16x32_bf16, lane = 16*c + r)
//   S^T = K Q^T : A = K chunk (rows = 16 keys, contraction = d), B = Q^T.  Query
//     row r sits in lane column r, keys 4c..4c+3 in the four accumulators: the
//     softmax statistics of a row live in lanes r, r+16, r+32, r+48.
//   O^T = V^T P^T : B = P^T is what the lane already holds (row r, keys
//     {4c..4c+3} of both 16-key halves); A = V^T needs per lane 8 keys x 1 value
//     column, which the transposing LDS read of gfx950 (ds_read_b64_tr_b16)
//     delivers from row-major V directly: per PV step two reads (one per
//     16-key half), no in-register transpose.  V rows are chunk-swizzled for
//     that read pattern like K rows are for theirs.  Step j yields value
//     columns 16j..16j+15 (lane (r, c): columns 16j+4c..16j+4c+3 of row r).
//     O^T keeps row r in lane column r too, so the running-max rescale is a
//     per-lane multiply -- and away from the mask no maximum is tracked at all
//     (exponentials against the reference the earlier chunks left, with the
//     tracked form as fallback; see compute_tile).
#include <atomic>

#include "common.h"

namespace specvlm {

#define SPECVLM_AS1 __attribute__((address_space(1)))
#define SPECVLM_AS3 __attribute__((address_space(3)))

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
    __bf16* part_o;          // [batch*H_kv][num_splits][rows_pad][D] unnormalised partial outputs (bf16: see the merge kernel)
    float* part_ml;          // [batch*H_kv][num_splits][rows_pad][2] (running max in log2 units, sum)
    int rows_pad;            // rows per partial slot: n_rgroups * (row blocks per workgroup) * 16
    int n_rgroups;           // groups of at most 4 row blocks that share a (head, split): one workgroup each
    int n_work;
    const uint64_t* block_mask;  // [sum q_len] tree masks of the block's queries, or null (chain)
    int balanced;            // batch mode: balanced pieces (see attn_balance) instead of uniform splits
    int max_wg;              // workgroups launched in balanced mode
    int tile_keys;           // keys per tile of the split kernel that runs (the unit of balanced mode)
    int32_t* seg_table;      // balanced mode: per (request, head) {first partial slot, pieces}, written by workgroup 0
};

constexpr int kChunkKeys = 32;       // keys per PV contraction step
constexpr int kMaxBalancedBatch = 64;   // (every workgroup walks the request lengths once)

// Tiles of request b in balanced mode; a request with nothing to do (no queries, or fewer keys
// than queries) has none.
__device__ __forceinline__ int attn_request_tiles(const AttnParams& p, int b, int tile_keys)
{
    const int ql = p.cu_q[b + 1] - p.cu_q[b], kvl = p.cu_kv[b + 1] - p.cu_kv[b];
    return (ql <= 0 || kvl < ql) ? 0 : (kvl + tile_keys - 1) / tile_keys;
}

struct AttnBalance { int64_t n_units; int n_groups; };

// Balanced mode deals TILES OF REQUESTS (all kv heads of a token range together) to groups of
// n_kv_heads workgroups, one workgroup per head: n_units = tiles over the batch, n_groups = groups
// that share them -- never more groups than units, so every group's run is non-empty and the groups
// that touch a request are consecutive.  The workgroups of a group walk the same token rows at the
// same time (one DRAM page serves all heads of a token-major cache), and with workgroup ids dealt to
// the XCDs round-robin a kv head stays on one XCD.
__device__ __forceinline__ AttnBalance attn_balance(const AttnParams& p, int tile_keys)
{
    int64_t n = 0;
    for (int b = 0; b < p.batch; ++b) n += attn_request_tiles(p, b, tile_keys);
    AttnBalance r;
    r.n_units = n;
    r.n_groups = (int)min((int64_t)(p.max_wg / p.n_kv_heads), n);
    return r;
}
constexpr int kMaxSplits = 256;
constexpr float kSumRedo = 0x1p100f;     // a lane's sum of one chunk at or above this (or NaN) is redone with the maximum tracked
constexpr int kMaxQueryBlock = 64;      // queries per request: a row's view of its block is one 64-bit mask
constexpr int kMaxDevices = 64;         // per-device host state (kernel attributes, scratch addresses)
constexpr int kTargetWorkgroups = 192;  // workgroups of a single-request launch

// s_waitcnt immediate (gfx9 encoding) that waits for vmcnt <= n only.
constexpr int vmcnt_imm(int n)
{
    return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8);
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(N));
}

// Workgroup barrier that does not drain the direct-to-LDS loads still in
// flight for younger stages (a fence would).  Ordering of this wave's own LDS
// traffic is handled by the s_waitcnt the compiler places before each use.
__device__ __forceinline__ void stage_barrier()
{
    __asm__ volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __asm__ volatile("" ::: "memory");
}

// Reductions over the four lanes r, r+16, r+32, r+48 that share a query row,
// with the VALU lane-swap instructions of gfx950 (no LDS crossbar round trip):
// v_permlane32_swap exchanges the upper 32 lanes of one operand with the lower
// 32 of the other, v_permlane16_swap the odd 16-lane rows with the even ones.
__device__ __forceinline__ float quad_max(float x)
{
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float quad_sum(float x)
{
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

constexpr int largest_divisor_le(int n, int cap)
{
    int best = 1;
    for (int d = 1; d <= cap; ++d) if (n % d == 0) best = d;
    return best;
}

// XOR applied to the 16-byte chunk index of value row `key` inside a tile.  The transposing read of
// one PV step touches, per 32 lanes, 8 consecutive keys x 32 contiguous bytes (two chunks 2j, 2j+1):
// with the pair index XORed by the key (d = 128: key mod 8; d = 64, two rows per 256 bytes: key/2
// mod 4) those 8 x 32 bytes fall on 64 distinct banks.
template <int D> __device__ __forceinline__ constexpr int v_swizzle(int key)
{
    return (D == 128) ? ((key & 7) << 1) : (((key >> 1) & 3) << 1);
}

// ds_read_b64_tr_b16: every lane hands in the address of 8 bytes (four 16-bit elements); inside each
// group of 16 lanes, lanes 4x..4x+3 together hold "row" x (16 elements), and lane o receives element o
// of rows 0..3.  Issued as assembly, with the wait below: as a builtin the compiler cannot tell the
// read from one that aliases the direct-to-LDS loads still in flight and drains them (vmcnt 0) first.
template <int OFFSET>
__device__ __forceinline__ u32x2 lds_read_tr16(uint32_t lds_addr)
{
    u32x2 v;
    __asm__ volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=&v"(v) : "v"(lds_addr), "n"(OFFSET));
    return v;
}

// Waits for this wave's LDS reads; the fragments pass through so that their uses stay behind the wait.
template <int N>
__device__ __forceinline__ void lds_wait_fragments(bf16x8 (&f)[N])
{
    static_assert(N == 4 || N == 8, "one fragment per 16 value columns");
    if constexpr (N == 8)
        __asm__ volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
    else
        __asm__ volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
}

// NLD: waves of a workgroup that only issue the direct-to-LDS loads (0: the compute waves issue them)
template <int D, int MB, int KS, int TK, int NS, int NLD, bool STREAM>
__global__ __launch_bounds__((MB * KS + NLD) * kWave)
void attn_split_kernel(const AttnParams p)
{
    constexpr int NW = MB * KS;                  // compute waves per workgroup (the loader waves come after them)
    constexpr bool SPLIT_ROLES = NLD > 0;
    constexpr int DJ = D / 16;                   // value columns per lane (8 or 4)
    constexpr int KK = D / 32;                   // MFMA steps over the head dimension
    constexpr int CH = D / 8;                    // 16-byte chunks per key row
    constexpr int ROW_BYTES = D * 2;
    constexpr int KEYS_PER_LOAD = kWave / CH;    // key rows one wave-wide load covers (4 or 8)
    constexpr int TILE_BYTES = TK * ROW_BYTES;   // one of K or V
    constexpr int LOADS_PER_MAT = TK / KEYS_PER_LOAD;
    constexpr int LOADS = 2 * LOADS_PER_MAT;     // wave-wide loads per stage (K then V)
    constexpr int LW = SPLIT_ROLES ? NLD : largest_divisor_le(LOADS, NW);   // waves that issue loads
    constexpr int LPW = LOADS / LW;              // loads per loader wave per stage
    static_assert(LOADS % LW == 0, "the loads of a stage must divide among the loader waves");
    constexpr int NCHUNK = TK / kChunkKeys;      // 32-key chunks per tile
    constexpr int LDS_STRIDE = D + 4;            // merge buffer row stride (floats)
    static_assert(NCHUNK % KS == 0, "chunks must divide among the key-split waves");
    static_assert(NS >= 2 && NS <= 5, "ring depth");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool is_loader = SPLIT_ROLES ? wave >= NW : wave < LW;
    const bool computes = SPLIT_ROLES ? wave < NW : true;
    const int lw = SPLIT_ROLES ? wave - NW : wave;   // loader index
    const int mb = wave % MB, ks = wave / MB;    // (compute waves)
    const int r = lane & 15, c = lane >> 4;

    extern __shared__ __align__(16) unsigned char smem[];
    // stage s: K tile at s*2*TILE_BYTES, V tile right after it

    // One piece of work: keys [k_begin, k_end) of (request b, kv head g) for all its query rows;
    // the result goes to partial slot slot0 (in units of rows), or straight to the output.
    auto piece = [&](const int b, const int g, const int row0, const int k_begin, const int k_end,
                     const int64_t slot0, const bool direct) {
    int q0 = 0, ql = p.q_len, kv0 = 0, kvl = p.kv_len;
    if (p.cu_q) { q0 = p.cu_q[b]; ql = p.cu_q[b + 1] - q0; }
    if (p.cu_kv) { kv0 = p.cu_kv[b]; kvl = p.cu_kv[b + 1] - kv0; }
    const int n_rows = p.group * ql;                // live query rows of this kv head

    // ---- this wave's Q fragments (B operand of S^T) ----
    // They travel HBM -> LDS -> registers like the tiles do (through the ring's last stage, which
    // no tile uses before the first barrier).  A load that returns into registers would make the
    // compiler guard those registers with waits that also drain the younger tile loads.
    bf16x8 qf[KK];
    int t_blk;                  // this lane's query row is the block's t_blk-th query
    unsigned char* q_stage = smem + (NS - 1) * (2 * TILE_BYTES) + wave * (KK * 1024);
    static_assert(MB * KS * KK * 1024 <= 2 * TILE_BYTES, "Q staging must fit in one ring stage");
    if (computes) {
        const int row = row0 + mb * 16 + r;
        const bool live = row < n_rows;             // padding rows read row 0: finite, never stored
        const int t = live ? row / p.group : 0;
        const int h = g * p.group + (live ? row % p.group : 0);
        t_blk = t;
        const __bf16* qp = p.q + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head + c * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)(qp + kk * 32),
                                             (SPECVLM_AS3 void*)(q_stage + kk * 1024), 16, 0, 0);
    }

    const char* kbase = reinterpret_cast<const char*>(p.k + (int64_t)kv0 * p.kv_tok + (int64_t)g * p.kv_head);
    const char* vbase = reinterpret_cast<const char*>(p.v + (int64_t)kv0 * p.kv_tok + (int64_t)g * p.kv_head);
    const uint32_t tok_bytes = (uint32_t)p.kv_tok * 2u;

    // ---- loader: wave-wide direct-to-LDS loads; load n of a stage covers
    // KEYS_PER_LOAD consecutive key rows of K (n < LOADS_PER_MAT) or of V ----
    const int ld_key = lane / CH;                   // key row inside the load
    const int ld_chunk = lane % CH;                 // LDS chunk slot inside the row
    auto issue_tile = [&](int tile, int stage) {
        const int base = k_begin + tile * TK;
        unsigned char* st = smem + stage * (2 * TILE_BYTES);
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int n = lw + LW * j;
            const bool is_v = n >= LOADS_PER_MAT;
            const int kl = (is_v ? n - LOADS_PER_MAT : n) * KEYS_PER_LOAD + ld_key;   // key inside the tile
            // rows past the split's end are masked in the compute: re-read its last row
            // (a cache hit) instead of pulling the neighbour split's keys from HBM
            const uint32_t key = (uint32_t)min(base + kl, k_end - 1);
            // K and V rows are chunk-swizzled so the operand reads spread over the banks: K for 16 keys x
            // one chunk per 16 lanes, V for the transposing read (8 keys x two neighbouring chunks per
            // 32 lanes, see v_swizzle)
            const int swz = is_v ? v_swizzle<D>(kl) : ((D == 128) ? (kl & 15) : ((kl >> 1) & 7));
            const int chunk = ld_chunk ^ swz;
            const char* src = (is_v ? vbase : kbase) + (key * tok_bytes + (uint32_t)chunk * 16u);
            unsigned char* dst = st + n * 1024;     // + lane * 16 by the hardware
            // a large cache is read once per launch: non-temporal, so it does not displace what is reused;
            // a small one (the draft's pruned cache, re-read every decode step) stays cacheable
            __builtin_amdgcn_global_load_lds((const SPECVLM_AS1 void*)src, (SPECVLM_AS3 void*)dst, 16, 0, STREAM ? 2 : 0);
        }
    };

    float m_run = -INFINITY, l_run = 0.f;
    floatx4 o_acc[DJ];
#pragma unroll
    for (int j = 0; j < DJ; ++j) o_acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // (a zero scale is taken as a vanishing one, so that a masked logit, -inf, times the scale stays -inf
    // instead of becoming NaN; every other logit still scales to 0)
    const float sc = fmaxf(p.scale_log2, 1e-30f);
    auto compute_tile = [&](int tile, int stage) {
        const unsigned char* kt_lds = smem + stage * (2 * TILE_BYTES);
        const unsigned char* vt_lds = kt_lds + TILE_BYTES;
#pragma unroll
        for (int cc = 0; cc < NCHUNK / KS; ++cc) {
            const int chunk = ks + cc * KS;
            const int base = k_begin + tile * TK + chunk * kChunkKeys;
            if (base >= k_end) break;
            const bool need_mask = (base + kChunkKeys > k_end) || (base + kChunkKeys > kvl - ql);
            // ---- S^T = K Q^T for 32 keys ----
            floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int x = kk * 4 + c;
                const int key0 = chunk * kChunkKeys + r, key1 = key0 + 16;
                const int sw0 = (D == 128) ? (key0 & 15) : ((key0 >> 1) & 7);
                const int sw1 = (D == 128) ? (key1 & 15) : ((key1 >> 1) & 7);
                const u32x4 k0 = *reinterpret_cast<const u32x4*>(kt_lds + key0 * ROW_BYTES + ((x ^ sw0) * 16));
                const u32x4 k1 = *reinterpret_cast<const u32x4*>(kt_lds + key1 * ROW_BYTES + ((x ^ sw1) * 16));
                s0 = mfma16(__builtin_bit_cast(bf16x8, k0), qf[kk], s0);
                s1 = mfma16(__builtin_bit_cast(bf16x8, k1), qf[kk], s1);
            }
            // The logits stay unscaled: the scale (> 0) is applied to the maximum once and rides in the
            // fused multiply-add that forms each exponent.
            float s[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { s[i] = s0[i]; s[4 + i] = s1[i]; }
            if (need_mask) {
                // Block keys this lane's query row may see (bit b = block key b).  Chain: the block is
                // causal, query t sees block keys 0..t; tree: the caller's ancestor mask, fetched here
                // (only the last chunks of a request get here) rather than held through the sweep.
                const uint64_t row_mask = p.block_mask ? p.block_mask[q0 + t_blk] : ((2ull << t_blk) - 1ull);
                const uint32_t mask_lo = (uint32_t)row_mask, mask_hi = (uint32_t)(row_mask >> 32);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int key = base + (i < 4 ? 4 * c + i : 16 + 4 * c + (i - 4));
                    const int bk = key - (kvl - ql);        // index inside the block (negative: context key)
                    const uint32_t word = (bk & 32) ? mask_hi : mask_lo;
                    const bool in_block_hidden = bk >= 0 && ((word >> (bk & 31)) & 1u) == 0u;
                    s[i] = (key >= k_end || in_block_hidden) ? -INFINITY : s[i];
                }
            }
            // V^T fragments of the lane's 8 keys (4c+i and 16+4c+i, i < 4) by the transposing LDS read:
            // the 16 lanes of quarter c hand in the rows of keys 4c + x (x = r/4; four lanes per key,
            // 8 bytes each, together columns 16j..16j+15) and lane r receives column 16j + r of the four
            // keys -- the A operand of step j with no in-register transpose.
            bf16x8 vf[DJ];
            {
                const int kl = chunk * kChunkKeys + 4 * c + (r >> 2);           // (the second half is 16 rows on)
                const int pair_swz = v_swizzle<D>(kl) >> 1;                     // same for kl + 16
                const uint32_t vrow = (uint32_t)(uintptr_t)(SPECVLM_AS3 const void*)(vt_lds + kl * ROW_BYTES + (r & 3) * 8);
#pragma unroll
                for (int j = 0; j < DJ; ++j) {
                    const uint32_t src = vrow + (uint32_t)((j ^ pair_swz) * 32);
                    const u32x2 lo = lds_read_tr16<0>(src);
                    const u32x2 hi = lds_read_tr16<16 * ROW_BYTES>(src);
                    vf[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
                }
            }
            // Away from the mask the running maximum is not tracked: the exponentials are taken against
            // the reference the earlier chunks left (a logit above it only makes its term larger than one),
            // which saves the maximum, its exchange over the quarter waves and the rescale test -- a
            // quarter of a chunk's VALU work.  A lane sum that is no longer a moderate finite number (a
            // logit 2^100 above the reference, or a reference not set yet) sends the wave through the
            // tracked form of the same chunk instead.
            floatx8 pv;
            bool settled = false;
            if (!need_mask && !__any(!(m_run > -INFINITY))) {
                float psum = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) { pv[i] = fast_exp2(fmaf(s[i], sc, -m_run)); psum += pv[i]; }
                if (!__any(!(psum < kSumRedo))) {
                    l_run += psum;
                    settled = true;
                }
            }
            if (!settled) {
                float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                                 fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
                mx = quad_max(mx) * sc;
                const float m_new = fmaxf(m_run, mx);
                const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = fast_exp2(m_run - m_ref);
                const bool rescale = m_new != m_run;
                m_run = m_new;
                float psum = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) { pv[i] = fast_exp2(fmaf(s[i], sc, -m_ref)); psum += pv[i]; }
                l_run = l_run * alpha + psum;
                if (__any(rescale)) {
#pragma unroll
                    for (int j = 0; j < DJ; ++j) o_acc[j] *= alpha;
                }
            }
            const bf16x8 pf = __builtin_convertvector(pv, bf16x8);
            // ---- O^T += V^T P^T ----
            lds_wait_fragments(vf);
#pragma unroll
            for (int j = 0; j < DJ; ++j) o_acc[j] = mfma16(vf[j], pf, o_acc[j]);
        }
    };

    // ---- ring of NS stages: NS-1 tiles in flight while one is consumed ----
    // The loader waves always start NS-1 tiles (a split shorter than that loads its last tile
    // again into a stage nobody reads), then every wave waits for its Q fragments, which are older
    // than any tile load, and takes them into registers.
    const int n_tiles = (k_end - k_begin + TK - 1) / TK;            // >= 1
    const int n_load = n_tiles > NS - 1 ? n_tiles : NS - 1;          // tiles as the loader counts them
    if constexpr (SPLIT_ROLES) {
    // Two loops, one per role (their registers do not add up); both pass the same barrier once per tile.
    if (is_loader) {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue_tile(s < n_tiles ? s : n_tiles - 1, s);
        int i = 0;
        do {
            // tiles issued after tile i so far: min(NS-2, n_load-1-i); each is LPW loads of a loader wave
            const int younger = min(NS - 2, n_load - 1 - i);
            wait_vmcnt<(NS - 2) * LPW>();
            if constexpr (NS >= 5) { if (younger <= 2) wait_vmcnt<2 * LPW>(); }
            if constexpr (NS >= 4) { if (younger <= 1) wait_vmcnt<1 * LPW>(); }
            if constexpr (NS >= 3) { if (younger <= 0) wait_vmcnt<0>(); }
            stage_barrier();                         // tile i landed for everyone; stage (i-1)%NS is free
            if (i + NS - 1 < n_load) issue_tile(i + NS - 1, (i + NS - 1) % NS);
        } while (++i < n_tiles);
        wait_vmcnt<0>();                             // (a short split's spare copies may still be landing)
    } else {
        wait_vmcnt<0>();                             // a compute wave's only loads: its Q fragments
        __asm__ volatile("" ::: "memory");
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qf[kk] = *reinterpret_cast<const bf16x8*>(q_stage + kk * 1024 + lane * 16);
        __asm__ volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): read before the stage is handed to the loaders
        __asm__ volatile("" ::: "memory");
        int i = 0;
        do {
            stage_barrier();
            compute_tile(i, i % NS);
        } while (++i < n_tiles);
    }
    } else {
    // Every wave computes and the first LW of them also issue the loads.  The loader waves always start
    // NS-1 tiles, then every wave waits for its Q fragments, which are older than any tile load.
    if (is_loader) {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue_tile(s < n_tiles ? s : n_tiles - 1, s);
        wait_vmcnt<(NS - 1) * LPW>();                // the Q loads are older than every tile load
    } else {
        wait_vmcnt<0>();
    }
    __asm__ volatile("" ::: "memory");
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
        qf[kk] = *reinterpret_cast<const bf16x8*>(q_stage + kk * 1024 + lane * 16);
    __asm__ volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): read before the stage is handed to the loader
    __asm__ volatile("" ::: "memory");
    int i = 0;
    do {
        // tiles issued after tile i so far: min(NS-2, n_load-1-i); each is LPW loads of a loader wave
        const int younger = min(NS - 2, n_load - 1 - i);
        wait_vmcnt<(NS - 2) * LPW>();
        if constexpr (NS >= 5) { if (younger <= 2) wait_vmcnt<2 * LPW>(); }
        if constexpr (NS >= 4) { if (younger <= 1) wait_vmcnt<1 * LPW>(); }
        if constexpr (NS >= 3) { if (younger <= 0) wait_vmcnt<0>(); }
        stage_barrier();                             // tile i landed for everyone; stage (i-1)%NS is free
        if (is_loader && i + NS - 1 < n_load) issue_tile(i + NS - 1, (i + NS - 1) % NS);
        compute_tile(i, i % NS);
    } while (++i < n_tiles);
    wait_vmcnt<0>();                                 // (a short split's spare copies may still be landing)
    }

    // ---- epilogue (the loader waves only keep the barriers of the exchange) ----
    if constexpr (KS == 1) { if (!computes) return; }
    l_run = quad_sum(l_run);
    const int row = row0 + mb * 16 + r;
    const int t_row = row / p.group, h_row = g * p.group + row % p.group;
    const int64_t slot = slot0 + row;
    if constexpr (KS == 1) {
        // lane (r, c) holds columns 16j + 4c .. 16j + 4c + 3 of its row in o_acc[j]: write them out directly
        if (direct) {
            if (row >= n_rows) return;
            const float inv = 1.f / l_run;
            __bf16* op = p.out + (int64_t)(q0 + t_row) * p.q_tok + (int64_t)h_row * p.q_head + 4 * c;
#pragma unroll
            for (int j = 0; j < DJ; ++j)
                *reinterpret_cast<bf16x4*>(op + 16 * j) = __builtin_convertvector(o_acc[j] * inv, bf16x4);
            if (p.lse && c == 0)
                p.lse[(int64_t)(q0 + t_row) * p.n_q_heads + h_row] = (m_run + fast_log2(l_run)) * kLn2;
        } else {
            __bf16* po = p.part_o + slot * D + 4 * c;
#pragma unroll
            for (int j = 0; j < DJ; ++j)
                *reinterpret_cast<bf16x4*>(po + 16 * j) = __builtin_convertvector(o_acc[j], bf16x4);
            if (c == 0) { p.part_ml[slot * 2] = m_run; p.part_ml[slot * 2 + 1] = l_run; }
        }
    } else {
        // The KS waves of a row block exchange their accumulators through LDS;
        // afterwards wave ks owns the column slice [ks*D/KS, (ks+1)*D/KS) of all
        // 16 rows, so every wave takes part in the final add and store.
        constexpr int SLICE = D / KS;                // columns per wave after the exchange
        constexpr int CPL = SLICE / 4;               // columns per lane (lane (r, c): c-th quarter)
        __syncthreads();                             // every wave is done with the ring
        float* sm_m = reinterpret_cast<float*>(smem);            // [NW][16]
        float* sm_l = sm_m + NW * 16;                            // [NW][16]
        float* sm_o = sm_l + NW * 16;                            // [NW][16][LDS_STRIDE]
        if (c == 0 && computes) sm_m[wave * 16 + r] = m_run;
        __syncthreads();
        float m_all = m_run;
#pragma unroll
        for (int kx = 0; kx < KS; ++kx) m_all = fmaxf(m_all, sm_m[(kx * MB + mb) * 16 + r]);
        const float f = fast_exp2(m_run - ((m_all == -INFINITY) ? 0.f : m_all));
        if (c == 0 && computes) sm_l[wave * 16 + r] = l_run * f;
        if (computes) {
            float* buf = sm_o + (wave * 16 + r) * LDS_STRIDE + 4 * c;
#pragma unroll
            for (int j = 0; j < DJ; ++j) *reinterpret_cast<floatx4*>(buf + 16 * j) = o_acc[j] * f;
        }
        __syncthreads();
        if (!computes) return;
        float l_all = 0.f;
#pragma unroll
        for (int kx = 0; kx < KS; ++kx) l_all += sm_l[(kx * MB + mb) * 16 + r];
        const int col0 = ks * SLICE + c * CPL;
        floatx4 acc[CPL / 4];
#pragma unroll
        for (int qd = 0; qd < CPL / 4; ++qd) acc[qd] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kx = 0; kx < KS; ++kx) {
            const float* buf = sm_o + ((kx * MB + mb) * 16 + r) * LDS_STRIDE + col0;
#pragma unroll
            for (int qd = 0; qd < CPL / 4; ++qd) acc[qd] += *reinterpret_cast<const floatx4*>(buf + 4 * qd);
        }
        if (direct) {
            if (row >= n_rows) return;
            const float inv = 1.f / l_all;
            __bf16* op = p.out + (int64_t)(q0 + t_row) * p.q_tok + (int64_t)h_row * p.q_head + col0;
#pragma unroll
            for (int qd = 0; qd < CPL / 4; ++qd)
                *reinterpret_cast<bf16x4*>(op + 4 * qd) = __builtin_convertvector(acc[qd] * inv, bf16x4);
            if (p.lse && c == 0 && ks == 0)
                p.lse[(int64_t)(q0 + t_row) * p.n_q_heads + h_row] = (m_all + fast_log2(l_all)) * kLn2;
        } else {
            __bf16* po = p.part_o + slot * D + col0;
#pragma unroll
            for (int qd = 0; qd < CPL / 4; ++qd) *reinterpret_cast<bf16x4*>(po + 4 * qd) = __builtin_convertvector(acc[qd], bf16x4);
            if (c == 0 && ks == 0) { p.part_ml[slot * 2] = m_all; p.part_ml[slot * 2 + 1] = l_all; }
        }
    }
    };   // piece

    if (!p.balanced) {
        // Uniform splits.  Dispatch order: the kv heads of one (request, row group, split) are neighbours.
        // Workgroups are dealt to the XCDs round-robin by id, so with 8 kv heads every split of head
        // g runs on XCD g: its partial results stay near that XCD, where the merge kernel (same
        // head-to-XCD order) finds them.  Token-major caches interleave the heads inside every token
        // row, so neighbours also walk the same DRAM pages at the same time.
        const int vid = blockIdx.x;
        const int g = vid % p.n_kv_heads, rest = vid / p.n_kv_heads;
        const int split = rest % p.num_splits;
        // more than 64 query rows per kv head: groups of MB row blocks, one workgroup each; the groups of
        // a (head, split) re-read its keys, as neighbours in time on one XCD (mostly from its L2)
        const int rg = (rest / p.num_splits) % p.n_rgroups;
        const int b = rest / (p.num_splits * p.n_rgroups);
        int ql = p.q_len, kvl = p.kv_len;
        if (p.cu_q) ql = p.cu_q[b + 1] - p.cu_q[b];
        if (p.cu_kv) kvl = p.cu_kv[b + 1] - p.cu_kv[b];
        if (ql <= 0 || kvl < ql) return;
        const int k_begin = split * p.split_keys;
        if (k_begin >= kvl) return;                     // the merge reads only the live splits
        const int bh = b * p.n_kv_heads + g;
        piece(b, g, rg * (MB * 16), k_begin, min(kvl, k_begin + p.split_keys),
              ((int64_t)bh * p.num_splits + split) * p.rows_pad, p.num_splits == 1);
        return;
    }

    // Balanced pieces for a batch.  The unit of work is one tile of one request (all kv heads); the
    // units are numbered request-major, then tile, and group j -- workgroups j*H .. j*H+H-1, one per
    // kv head -- takes the contiguous run [j*T/G, (j+1)*T/G).  A run that crosses from one request
    // into the next is cut into pieces there; piece (group j, request b) of head g owns partial slot
    // (j + b)*H + g, unique because from one piece to the next exactly one of j and b grows.  Every
    // workgroup derives the same numbers from the request lengths, as the merge kernel does.
    const AttnBalance bal = attn_balance(p, TK);
    const int H = p.n_kv_heads;
    const int w = blockIdx.x;
    if (w == 0) {
        // the merge kernel's view of the decomposition: for every (request, head) its first partial
        // slot and the number of pieces (the groups that touch a request are consecutive; the group
        // that owns unit x is the largest j with j*T/G <= x)
        for (int seg = threadIdx.x; seg < p.batch * H; seg += (MB * KS + NLD) * kWave) {
            const int sb = seg / H, sg = seg % H;
            int64_t first = 0;
            for (int bb = 0; bb < sb; ++bb) first += attn_request_tiles(p, bb, TK);
            const int tiles = attn_request_tiles(p, sb, TK);
            int j_first = 0, live = 0;
            if (tiles > 0) {
                j_first = (int)(((first + 1) * bal.n_groups - 1) / bal.n_units);
                live = (int)(((first + tiles) * bal.n_groups - 1) / bal.n_units) - j_first + 1;
            }
            p.seg_table[2 * seg] = (j_first + sb) * H + sg;
            p.seg_table[2 * seg + 1] = live;
        }
    }
    const int j = w / H, g = w % H;
    if (j >= bal.n_groups) return;
    int64_t x = (int64_t)j * bal.n_units / bal.n_groups;
    const int64_t x_end = (int64_t)(j + 1) * bal.n_units / bal.n_groups;
    int b = 0;
    int64_t base = 0;                                   // first unit of request b
    while (x < x_end) {
        int tiles = attn_request_tiles(p, b, TK);
        while (x >= base + tiles) {
            base += tiles;
            ++b;
            tiles = attn_request_tiles(p, b, TK);
        }
        const int t = (int)(x - base);
        const int n = (int)min((int64_t)(tiles - t), x_end - x);
        const int kvl = p.cu_kv[b + 1] - p.cu_kv[b];
        piece(b, g, 0, t * TK, min(kvl, (t + n) * TK), (int64_t)((j + b) * H + g) * p.rows_pad, false);
        x += n;
        __syncthreads();                                // the next piece reuses the ring and the exchange buffer
    }
}

// Merge of the split partials: o = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s.
// The partial outputs travel as bf16 (the running maxima and sums stay fp32): each is rounded once, by
// at most 2^-9 of its own size, and the merged row is a convex combination of them, so the detour adds
// at most one more rounding of the size the bf16 output carries anyway, and it halves the bytes that
// the two kernels exchange.
// One workgroup per (kv head, query row); thread (grp, col) folds the splits grp, grp + GROUPS, ...
// for 4 output columns.  Every load of the first PRE splits per thread is issued up front, so the
// kernel costs one memory round trip; each group folds its splits against its own maximum and a
// single barrier later group 0 combines the GROUPS partial results.
// Twelve groups (two loads per thread at the usual 24 splits per head) measured best: 16.3 us per 72B
// layer against 16.7 with 8 groups, 16.35 with 16, 16.85 with 24 and 17.5 with 32; several rows per
// workgroup are slower as well (16.9 with two, 17.2 with four).
template <int D, int PRE, int THREADS>
__global__ __launch_bounds__(THREADS)
void attn_merge_kernel(const AttnParams p)
{
    constexpr int TPR = D / 4;                       // threads that cover one row of D columns
    constexpr int GROUPS = THREADS / TPR;            // split groups working in parallel
    __shared__ float s_m[GROUPS], s_l[GROUPS];
    __shared__ __align__(16) float s_acc[GROUPS][D];
    // (request, kv head) fastest: workgroup id modulo the XCD count follows the kv head, as in the split kernel
    const int nbh = p.batch * p.n_kv_heads;
    const int bh = blockIdx.x % nbh, row = blockIdx.x / nbh;
    const int b = bh / p.n_kv_heads, g = bh % p.n_kv_heads;
    int q0 = 0, ql = p.q_len, kvl = p.kv_len;
    if (p.cu_q) { q0 = p.cu_q[b]; ql = p.cu_q[b + 1] - q0; }
    if (p.cu_kv) { kvl = p.cu_kv[b + 1] - p.cu_kv[b]; }
    if (ql <= 0 || kvl < ql || row >= p.group * ql) return;
    // the partial slots of this (request, head) are consecutive: splits 0..live-1
    const int live = min(p.num_splits, (kvl + p.split_keys - 1) / p.split_keys);
    const int64_t slot0 = (int64_t)bh * p.num_splits * p.rows_pad + row;
    const int tid = threadIdx.x;
    const int grp = tid / TPR, col = (tid % TPR) * 4;

    float m_i[PRE], l_i[PRE];
    floatx4 ov[PRE];
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const int s = grp + GROUPS * i;
        m_i[i] = -INFINITY; l_i[i] = 0.f; ov[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (s < live) {
            const int64_t slot = slot0 + (int64_t)s * p.rows_pad;
            const float* ml = p.part_ml + slot * 2;          // the same address across the group: one transaction
            m_i[i] = ml[0]; l_i[i] = ml[1];
            ov[i] = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(p.part_o + slot * D + col), floatx4);
        }
    }
    float m_loc = m_i[0];
#pragma unroll
    for (int i = 1; i < PRE; ++i) m_loc = fmaxf(m_loc, m_i[i]);
    float m_ref = (m_loc == -INFINITY) ? 0.f : m_loc;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    float l_loc = 0.f;
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const float w = fast_exp2(m_i[i] - m_ref);           // 0 for an absent or empty split
        acc += w * ov[i];
        l_loc += w * l_i[i];
    }
    for (int s = grp + GROUPS * PRE; s < live; s += GROUPS) {   // more splits than the prefetch covers
        const int64_t slot = slot0 + (int64_t)s * p.rows_pad;
        const float m_s = p.part_ml[slot * 2], l_s = p.part_ml[slot * 2 + 1];
        const floatx4 o_s = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(p.part_o + slot * D + col), floatx4);
        const float m_new = fmaxf(m_loc, m_s);
        const float r_new = (m_new == -INFINITY) ? 0.f : m_new;
        const float f_old = fast_exp2(m_loc - r_new), f_s = fast_exp2(m_s - r_new);
        acc = acc * f_old + f_s * o_s;
        l_loc = l_loc * f_old + f_s * l_s;
        m_loc = m_new;
    }
    *reinterpret_cast<floatx4*>(&s_acc[grp][col]) = acc;
    if (col == 0) { s_m[grp] = m_loc; s_l[grp] = l_loc; }
    __syncthreads();
    if (grp != 0) return;
    float m = s_m[0];
#pragma unroll
    for (int gg = 1; gg < GROUPS; ++gg) m = fmaxf(m, s_m[gg]);
    m_ref = (m == -INFINITY) ? 0.f : m;
    floatx4 tot = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int gg = 0; gg < GROUPS; ++gg) {
        const float f = fast_exp2(s_m[gg] - m_ref);
        tot += f * *reinterpret_cast<const floatx4*>(&s_acc[gg][col]);
        l += f * s_l[gg];
    }
    tot *= 1.f / l;
    const int t = row / p.group, h = g * p.group + row % p.group;
    __bf16* op = p.out + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head + col;
    *reinterpret_cast<bf16x4*>(op) = __builtin_convertvector(tot, bf16x4);
    if (p.lse && col == 0)
        p.lse[(int64_t)(q0 + t) * p.n_q_heads + h] = (m + fast_log2(l)) * kLn2;
}

// Merge for the balanced decomposition, where a (request, head) has only a handful of pieces: each
// group of D/4 threads merges one query row on its own, with the loads of up to PRE pieces in
// flight together, so a workgroup finishes 256 / (D/4) rows and no cross-thread combine is needed.
template <int D, int PRE>
__global__ __launch_bounds__(256)
void attn_merge_rows_kernel(const AttnParams p)
{
    constexpr int TPR = D / 4;
    constexpr int GROUPS = 256 / TPR;
    const int nbh = p.batch * p.n_kv_heads;
    const int bh = blockIdx.x % nbh;
    const int b = bh / p.n_kv_heads, g = bh % p.n_kv_heads;
    const int tid = threadIdx.x;
    const int row = (blockIdx.x / nbh) * GROUPS + tid / TPR, col = (tid % TPR) * 4;
    int q0 = 0, ql = p.q_len, kvl = p.kv_len;
    if (p.cu_q) { q0 = p.cu_q[b]; ql = p.cu_q[b + 1] - q0; }
    if (p.cu_kv) { kvl = p.cu_kv[b + 1] - p.cu_kv[b]; }
    if (ql <= 0 || kvl < ql || row >= p.group * ql) return;
    const int live = p.seg_table[2 * bh + 1];
    const int64_t slot0 = (int64_t)p.seg_table[2 * bh] * p.rows_pad + row;
    float m = -INFINITY, l = 0.f;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < live; s0 += PRE) {
        float m_i[PRE], l_i[PRE];
        floatx4 ov[PRE];
#pragma unroll
        for (int i = 0; i < PRE; ++i) {
            m_i[i] = -INFINITY; l_i[i] = 0.f; ov[i] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (s0 + i < live) {
                const int64_t slot = slot0 + (int64_t)(s0 + i) * p.n_kv_heads * p.rows_pad;   // the next group's piece
                m_i[i] = p.part_ml[slot * 2]; l_i[i] = p.part_ml[slot * 2 + 1];
                ov[i] = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(p.part_o + slot * D + col), floatx4);
            }
        }
        float m_new = m;
#pragma unroll
        for (int i = 0; i < PRE; ++i) m_new = fmaxf(m_new, m_i[i]);
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float f_old = fast_exp2(m - m_ref);
        acc *= f_old; l *= f_old;
#pragma unroll
        for (int i = 0; i < PRE; ++i) {
            const float w = fast_exp2(m_i[i] - m_ref);       // 0 for an absent or empty piece
            acc += w * ov[i];
            l += w * l_i[i];
        }
        m = m_new;
    }
    acc *= 1.f / l;
    const int t = row / p.group, h = g * p.group + row % p.group;
    __bf16* op = p.out + (int64_t)(q0 + t) * p.q_tok + (int64_t)h * p.q_head + col;
    *reinterpret_cast<bf16x4*>(op) = __builtin_convertvector(acc, bf16x4);
    if (p.lse && col == 0)
        p.lse[(int64_t)(q0 + t) * p.n_q_heads + h] = (m + fast_log2(l)) * kLn2;
}

// ---------------------------------------------------------------- host side ----
// A batch whose split count is left to the library is cut into balanced pieces by the kernels
// themselves (they know the request lengths; the host only knows their maximum).
static bool attn_is_balanced(int batch, int num_splits, int n_kv_heads, int rows)
{
    return batch > 1 && batch <= kMaxBalancedBatch && num_splits == 0 && n_kv_heads <= kNumCu && rows <= 64;
}

// Query rows of a kv head beyond 64 (long chains, draft trees) are cut into groups of equal size,
// at most 4 row blocks of 16 each: n groups, mb row blocks per group.
static void attn_row_groups(int rows, int* n_groups, int* mb)
{
    const int blocks = (rows + 15) / 16;
    *n_groups = (blocks + 3) / 4;
    *mb = (blocks + *n_groups - 1) / *n_groups;
}

static int choose_splits(int batch, int kv_len, int n_kv_heads, int n_rgroups, int num_splits)
{
    const int max_by_len = (kv_len + 127) / 128;              // at least two tiles per split
    int s = num_splits;
    if (s <= 0) {
        const int heads = batch * n_kv_heads * n_rgroups;
        // One request: a single round of workgroups, about three per four CUs.  Every workgroup then
        // streams the same share from start to end and HBM is saturated well before all CUs are
        // busy; more, smaller splits only add partial results and rounds (measured on 8 kv heads:
        // 131K keys run at 6.2 TB/s with 24 or 32 splits per head, 4.7 TB/s with 128; 33K keys at
        // 4.9 TB/s with 24, 4.2 TB/s with 32).
        s = (kTargetWorkgroups + heads - 1) / heads;
        // (with several row groups per head the sweep is bound by arithmetic, not HBM: as many workgroups
        // as fit in one round on the 256 CUs, never one more)
        if (n_rgroups > 1) s = kNumCu / heads;
        if (batch > 1) {
            // Batches too large for the balanced decomposition: cap a split at 2048 keys so that
            // long and short requests decompose into similar pieces the dispatcher can balance,
            // and make a launch of several rounds a whole number of rounds of 2 x 256 workgroups.
            const int by_len = (kv_len + 2047) / 2048;
            if (by_len > s) s = by_len;
            const int slots = 2 * kNumCu;
            if (heads * s > slots && slots % heads == 0) {
                const int unit = slots / heads;
                s = ((s + unit / 2) / unit) * unit;
                if (s < unit) s = unit;
            }
        }
    }
    if (s > max_by_len) s = max_by_len;
    if (s > kMaxSplits) s = kMaxSplits;
    if (s < 1) s = 1;
    return s;
}

template <int D, int MB, int KS, int TK, int NS, int NLD, bool STREAM>
static int launch_attn_s(const AttnParams& p, hipStream_t stream)
{
    constexpr int NW = MB * KS;
    constexpr size_t ring = (size_t)NS * 2 * TK * D * 2;
    constexpr size_t merge = KS > 1 ? sizeof(float) * (size_t)(2 * NW * 16 + NW * 16 * (D + 4)) : 0;
    constexpr size_t lds = ring > merge ? ring : merge;
    if (lds > 64 * 1024) {
        // the attribute belongs to the kernel as loaded on one device: raise it once per device
        static std::atomic<bool> raised[kMaxDevices];
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECVLM_ELAUNCH;
        if (!raised[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_split_kernel<D, MB, KS, TK, NS, NLD, STREAM>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                return SPECVLM_ELAUNCH;
            raised[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((attn_split_kernel<D, MB, KS, TK, NS, NLD, STREAM>), dim3(p.n_work), dim3((NW + NLD) * kWave),
                       lds, stream, p);
    return launch_status();
}

// From this size per launch on, the cache is streamed with non-temporal loads: its lines would
// only push the split partials (which the merge re-reads) and other reusable data out of the L2.
// Smaller caches (a draft's pruned cache, re-read at every decode step) stay cacheable.
constexpr int64_t kStreamBytes = 8ll << 20;

template <int D, int MB, int KS, int TK, int NS, int NLD>
static int launch_attn(const AttnParams& p, hipStream_t stream)
{
    const int64_t kv_bytes = 2ll * p.batch * p.n_kv_heads * (int64_t)p.kv_len * D * 2;
    return kv_bytes >= kStreamBytes ? launch_attn_s<D, MB, KS, TK, NS, NLD, true>(p, stream)
                                    : launch_attn_s<D, MB, KS, TK, NS, NLD, false>(p, stream);
}

template <int D>
static int launch_attn_d(const AttnParams& p, int mb, hipStream_t stream)
{

    // (key-split waves, tile keys, ring depth, loader waves) per row-block count; the ring
    // holds NS * 2 * TK * D * 2 bytes of LDS.  The single-query decode keeps its four waves (loading and
    // computing): on the draft's small cache the four extra waves cost more at workgroup start-up than
    // they save (6.7 against 6.4 us per layer).
    switch (mb) {
        case 1: return launch_attn<D, 1, 4, 128, 2, 0>(p, stream);
        case 2: return launch_attn<D, 2, 2, 64, 3, 4>(p, stream);
        case 3: return launch_attn<D, 3, 2, 64, 3, 2>(p, stream);   // (two loaders: 16.7 against 17.0 us with four)
        case 4: return launch_attn<D, 4, 2, 64, 3, 4>(p, stream);
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
    if (q_len > kMaxQueryBlock) return 0;
    int n_rgroups, mb;
    attn_row_groups(rows, &n_rgroups, &mb);
    const int rows_pad = n_rgroups * mb * 16;
    size_t slots;
    if (attn_is_balanced(batch, num_splits, n_kv_heads, rows)) {
        slots = (size_t)(kNumCu + batch * n_kv_heads) * rows_pad;
        return align256(slots * head_dim * sizeof(__bf16)) + align256(slots * 2 * sizeof(float)) +
               align256((size_t)batch * n_kv_heads * 2 * sizeof(int32_t));
    } else {
        const int splits = choose_splits(batch, kv_len, n_kv_heads, n_rgroups, num_splits);
        if (splits == 1) return 256;
        slots = (size_t)batch * n_kv_heads * splits * rows_pad;
    }
    return align256(slots * head_dim * sizeof(__bf16)) + align256(slots * 2 * sizeof(float));
}

static int attn_impl(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    const uint64_t* block_mask, void* out, float* lse, int num_splits,
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
    if (q_len > kMaxQueryBlock) return SPECVLM_EUNSUPPORTED;
    // per-lane key offsets are 32-bit byte offsets from the request's first row
    if (kv_tok_stride <= 0 || (int64_t)kv_len * kv_tok_stride * 2 >= ((int64_t)1 << 32))
        return SPECVLM_EUNSUPPORTED;
    int n_rgroups, mb;
    attn_row_groups(rows, &n_rgroups, &mb);

    AttnParams p;
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v;
    p.out = (__bf16*)out; p.lse = lse;
    p.q_tok = q_tok_stride; p.q_head = q_head_stride;
    p.kv_tok = kv_tok_stride; p.kv_head = kv_head_stride;
    p.cu_q = cu_q; p.cu_kv = cu_kv; p.block_mask = block_mask;
    p.batch = batch; p.q_len = q_len; p.kv_len = kv_len;
    p.n_q_heads = n_q_heads; p.n_kv_heads = n_kv_heads; p.group = group;
    p.scale_log2 = softmax_scale * kLog2e;
    p.balanced = attn_is_balanced(batch, num_splits, n_kv_heads, rows) ? 1 : 0;
    p.max_wg = kNumCu;
    p.tile_keys = mb == 1 ? 128 : 64;                 // TK of the launch shape chosen below
    p.num_splits = p.balanced ? 2 : choose_splits(batch, kv_len, n_kv_heads, n_rgroups, num_splits);
    p.split_keys = (kv_len + p.num_splits - 1) / p.num_splits;
    p.rows_pad = n_rgroups * mb * 16;
    p.n_rgroups = n_rgroups;
    p.n_work = p.balanced ? p.max_wg : batch * n_kv_heads * p.num_splits * n_rgroups;
    p.part_o = nullptr; p.part_ml = nullptr; p.seg_table = nullptr;
    if (p.num_splits > 1) {
        const size_t need = specvlm_decode_attn_workspace_bytes(batch, q_len, kv_len, n_q_heads,
                                                                n_kv_heads, head_dim, num_splits);
        if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SPECVLM_EWORKSPACE;
        const size_t slots = p.balanced ? (size_t)(p.max_wg + batch * n_kv_heads) * p.rows_pad
                                        : (size_t)batch * n_kv_heads * p.num_splits * p.rows_pad;
        p.part_o = (__bf16*)workspace;
        p.part_ml = (float*)((char*)workspace + align256(slots * head_dim * sizeof(__bf16)));
        p.seg_table = (int32_t*)((char*)p.part_ml + align256(slots * 2 * sizeof(float)));   // (used in balanced mode)
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = head_dim == 128 ? launch_attn_d<128>(p, mb, s) : launch_attn_d<64>(p, mb, s);
    if (rc != SPECVLM_OK) return rc;
    if (p.balanced) {
        const int per_wg = 256 / (head_dim / 4);
        dim3 grid((rows + per_wg - 1) / per_wg * batch * n_kv_heads);
        if (head_dim == 128) hipLaunchKernelGGL((attn_merge_rows_kernel<128, 8>), grid, dim3(256), 0, s, p);
        else                 hipLaunchKernelGGL((attn_merge_rows_kernel<64, 8>), grid, dim3(256), 0, s, p);
        rc = launch_status();
    } else if (p.num_splits > 1) {
        dim3 grid(rows * batch * n_kv_heads);
        if (head_dim == 128) hipLaunchKernelGGL((attn_merge_kernel<128, 3, 384>), grid, dim3(384), 0, s, p);
        else                 hipLaunchKernelGGL((attn_merge_kernel<64, 3, 192>), grid, dim3(192), 0, s, p);
        rc = launch_status();
    }
    return rc;
}

extern "C" int specvlm_decode_attn(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    void* out, float* lse, int num_splits,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_impl(q, q_tok_stride, q_head_stride, k, v, kv_tok_stride, kv_head_stride, cu_q, cu_kv,
                     batch, q_len, kv_len, n_q_heads, n_kv_heads, head_dim, softmax_scale, nullptr,
                     out, lse, num_splits, workspace, workspace_bytes, stream);
}

// ---- the variant that takes no workspace ----
// Scratch for callers that cannot allocate or pass one (code under HIP graph capture, serving loops
// that own no spare device memory).  Every device that loads the library holds its own copy of this
// array until the process ends; the name below is a host-side handle, the device address is looked
// up once per device.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECVLM_ELAUNCH;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SPECVLM_ELAUNCH;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // (every thread looks up the same address)
    }
    *out = ptr;
    return SPECVLM_OK;
}

extern "C" size_t specvlm_decode_attn_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int specvlm_decode_attn_static(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    void* out, float* lse, int num_splits, void* stream)
{
    // the shape decides how much scratch the kernels use; a shape the array cannot hold is refused
    // (a shape the workspace query itself rejects, size 0, is left to the argument checks below)
    const size_t need = specvlm_decode_attn_workspace_bytes(batch, q_len, kv_len, n_q_heads, n_kv_heads,
                                                            head_dim, num_splits);
    if (need > kStaticScratchBytes) return SPECVLM_EWORKSPACE;
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != SPECVLM_OK) return rc;
    return attn_impl(q, q_tok_stride, q_head_stride, k, v, kv_tok_stride, kv_head_stride, cu_q, cu_kv,
                     batch, q_len, kv_len, n_q_heads, n_kv_heads, head_dim, softmax_scale, nullptr,
                     out, lse, num_splits, ptr, kStaticScratchBytes, stream);
}

extern "C" int specvlm_tree_attn(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    const uint64_t* ancestor_mask, void* out, float* lse, int num_splits,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ancestor_mask && batch > 0 && q_len > 0) return SPECVLM_EINVAL;
    if (q_len > 64) return SPECVLM_EUNSUPPORTED;
    return attn_impl(q, q_tok_stride, q_head_stride, k, v, kv_tok_stride, kv_head_stride, cu_q, cu_kv,
                     batch, q_len, kv_len, n_q_heads, n_kv_heads, head_dim, softmax_scale, ancestor_mask,
                     out, lse, num_splits, workspace, workspace_bytes, stream);
}
