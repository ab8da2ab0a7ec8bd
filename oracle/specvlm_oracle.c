/*
 * CPU oracle for the SpecVLM speculative-decode hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 loops that write out what each
 * step of the path computes, so that a reader can check them against the
 * paper by eye.  Nothing here is used by the product (the HIP library); the
 * two share no code.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it.
 *
 * bf16 inputs arrive as uint16 bit patterns and are widened exactly to fp64.
 * All tensors are dense, row-major, one request per call:
 *     q    [n_q,  H_q,  d]
 *     k, v [n_kv, H_kv, d]
 * q head h reads kv head h / (H_q / H_kv)  (grouped-query attention).
 *
 * The only parallelism is an OpenMP "for" over (head, query) pairs; there is
 * no blocking, fusion or reordering inside a pair.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_f64(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double dot_bf16(const uint16_t* a, const uint16_t* b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += bf16_to_f64(a[c]) * bf16_to_f64(b[c]);
    return s;
}

/* ------------------------------------------------------------------------
 * Decode / verify attention  (Sec. 2.1: the draft decodes one token over its
 * cache; the target verifies gamma drafted tokens in one parallel forward).
 *
 * The verify block is the last committed token followed by the gamma drafted
 * tokens: q_len = gamma + 1 queries whose own K/V rows are already the last
 * q_len rows of the cache.  Query t sees keys j <= kv_len - q_len + t, which
 * is causal inside the block; q_len = 1 is plain decode.
 *
 *   o[t,h,:] = sum_j softmax_j(scale * q[t,h] . k[j,g]) * v[j,g,:]
 *   lse[t,h] = log sum_j exp(scale * q[t,h] . k[j,g])
 * ---------------------------------------------------------------------- */
int oracle_decode_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                       int q_len, int kv_len, int n_q_heads, int n_kv_heads, int d,
                       double scale, double* out /* [q_len,H_q,d] */,
                       double* lse /* [q_len,H_q] or NULL */)
{
    if (q_len < 0 || kv_len < q_len || n_kv_heads < 1 || n_q_heads % n_kv_heads) return -1;
    const int group = n_q_heads / n_kv_heads;
    const long rows = (long)q_len * n_q_heads;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        const int t = (int)(r / n_q_heads), h = (int)(r % n_q_heads), g = h / group;
        const int last = kv_len - q_len + t;        /* last visible key, inclusive */
        const uint16_t* qv = q + ((long)t * n_q_heads + h) * d;
        double* s = (double*)malloc(sizeof(double) * (size_t)(last + 1));
        if (!s) { failed = 1; continue; }
        double m = -INFINITY;
        for (int j = 0; j <= last; ++j) {
            s[j] = scale * dot_bf16(qv, k + ((long)j * n_kv_heads + g) * d, d);
            if (s[j] > m) m = s[j];
        }
        double z = 0.0;
        for (int j = 0; j <= last; ++j) z += exp(s[j] - m);
        double* o = out + r * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j <= last; ++j) {
            const double p = exp(s[j] - m) / z;
            const uint16_t* vv = v + ((long)j * n_kv_heads + g) * d;
            for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f64(vv[c]);
        }
        if (lse) lse[r] = m + log(z);
        free(s);
    }
    return failed ? -2 : 0;
}

/* ------------------------------------------------------------------------
 * Token scores  (Sec. 3.1, Eq. 4 and Eq. 5).
 *
 * G is the language-query x video-key block of the verifier's attention
 * matrix M; a_j is the mean of column j of G over the language queries, then
 * over heads.  Text query i sits at absolute position text_pos0 + i and sees
 * keys j <= text_pos0 + i.
 *
 * norm_mode 0: M is the full causal softmax (normalised over every visible
 *              key, video or not) and G is its video slice.
 * norm_mode 1: the softmax is taken over the visible video keys only.
 *
 *   scores[j] = beta * scores[j] + (1/(H_q*L)) * sum_h sum_i G[h,i,j]
 *
 * row_lse (optional, [L,H_q]) receives log of each row's normaliser.
 * ---------------------------------------------------------------------- */
int oracle_score(const uint16_t* q_text, const uint16_t* k,
                 int n_text, int n_keys, int video_start, int n_video, int text_pos0,
                 int n_q_heads, int n_kv_heads, int d, double scale, int norm_mode,
                 double beta, double* scores /* [n_video], in/out */,
                 double* row_lse /* [n_text,H_q] or NULL */)
{
    if (n_text < 0 || n_video < 0 || video_start < 0 || video_start + n_video > n_keys ||
        n_kv_heads < 1 || n_q_heads % n_kv_heads || (norm_mode != 0 && norm_mode != 1))
        return -1;
    const int group = n_q_heads / n_kv_heads;
    /* one column-sum vector per (query, head) row would be too large; keep one
       per head and add the rows of a head in query order. */
    double* per_head = (double*)calloc((size_t)n_q_heads * (size_t)(n_video > 0 ? n_video : 1),
                                       sizeof(double));
    if (!per_head) return -2;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < n_q_heads; ++h) {
        const int g = h / group;
        double* acc = per_head + (long)h * n_video;
        double* s = (double*)malloc(sizeof(double) * (size_t)(n_keys > 0 ? n_keys : 1));
        if (!s) { failed = 1; continue; }
        for (int i = 0; i < n_text; ++i) {
            const uint16_t* qv = q_text + ((long)i * n_q_heads + h) * d;
            int last = text_pos0 + i;
            if (last > n_keys - 1) last = n_keys - 1;
            const int lo = norm_mode ? video_start : 0;
            int hi = norm_mode ? video_start + n_video - 1 : last;   /* inclusive */
            if (hi > last) hi = last;
            double m = -INFINITY, z = 0.0;
            for (int j = lo; j <= hi; ++j) {
                s[j] = scale * dot_bf16(qv, k + ((long)j * n_kv_heads + g) * d, d);
                if (s[j] > m) m = s[j];
            }
            for (int j = lo; j <= hi; ++j) z += exp(s[j] - m);
            if (row_lse) row_lse[(long)i * n_q_heads + h] = (hi >= lo) ? m + log(z) : -INFINITY;
            for (int jv = 0; jv < n_video; ++jv) {
                const int j = video_start + jv;
                if (j > last || j < lo || j > hi) continue;
                acc[jv] += exp(s[j] - m) / z;
            }
        }
        free(s);
    }
    if (!failed) {
        const double denom = (double)n_q_heads * (double)n_text;
        for (int jv = 0; jv < n_video; ++jv) {
            double a = 0.0;
            for (int h = 0; h < n_q_heads; ++h) a += per_head[(long)h * n_video + jv];
            a = denom > 0 ? a / denom : 0.0;
            scores[jv] = (beta != 0.0 ? beta * scores[jv] : 0.0) + a;
        }
    }
    free(per_head);
    return failed ? -2 : 0;
}

/* ------------------------------------------------------------------------
 * Two-stage selection  (Sec. 3.2, Stage I and Stage II, Eq. 7).
 *
 * Stage I keeps V_R, the k highest-scoring video tokens (the paper sizes V_R
 * by cumulative mass, Eq. 6 -- see oracle_top_p_count -- here k is given).
 * Equal scores are ordered by lower token index first; -0.0 counts as +0.0;
 * NaN orders below every number.
 * Stage II walks the remaining tokens V \ V_R in raster order (frame-major,
 * then row-major on the frame's grid) and keeps U = B - k of them at the
 * fixed fractional interval I = R/U, R = n - k: the tokens of remainder rank
 * floor(t * R / U), t = 0..U-1.
 * Output: V_R u V_U ascending; from_topk marks members of V_R.
 * ---------------------------------------------------------------------- */
typedef struct { float key; int32_t idx; } scored_t;

static int score_rank(float x)   /* 0 for NaN (lowest), 1 for numbers */
{
    return isnan(x) ? 0 : 1;
}

static int cmp_desc(const void* pa, const void* pb)
{
    const scored_t* a = (const scored_t*)pa;
    const scored_t* b = (const scored_t*)pb;
    const int ra = score_rank(a->key), rb = score_rank(b->key);
    if (ra != rb) return rb - ra;                 /* numbers before NaN */
    if (ra == 1) {
        if (a->key > b->key) return -1;
        if (a->key < b->key) return 1;            /* -0.0 == +0.0 compares equal */
    }
    return (a->idx > b->idx) - (a->idx < b->idx); /* lower index first */
}

int oracle_select(const float* scores, int n_video, int k_top, int keep_budget,
                  int32_t* keep_idx /* [keep_budget] */, uint8_t* from_topk /* or NULL */)
{
    if (n_video < 0 || k_top < 0 || k_top > keep_budget || keep_budget > n_video) return -1;
    if (keep_budget == 0) return 0;
    scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)n_video);
    uint8_t* mark = (uint8_t*)calloc((size_t)n_video, 1);     /* 1 = V_R, 2 = V_U */
    int32_t* rem = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_video);
    if (!order || !mark || !rem) { free(order); free(mark); free(rem); return -2; }
    for (int j = 0; j < n_video; ++j) { order[j].key = scores[j]; order[j].idx = j; }
    qsort(order, (size_t)n_video, sizeof(scored_t), cmp_desc);
    for (int r = 0; r < k_top; ++r) mark[order[r].idx] = 1;
    int64_t R = 0;
    for (int j = 0; j < n_video; ++j) if (!mark[j]) rem[R++] = j;
    const int64_t U = (int64_t)keep_budget - k_top;
    for (int64_t t = 0; t < U; ++t) mark[rem[(t * R) / U]] = 2;
    int m = 0;
    for (int j = 0; j < n_video; ++j)
        if (mark[j]) {
            keep_idx[m] = j;
            if (from_topk) from_topk[m] = (uint8_t)(mark[j] == 1);
            ++m;
        }
    free(order); free(mark); free(rem);
    return m == keep_budget ? 0 : -3;
}

/* Stage I's own size rule (Eq. 6): the smallest c such that the c largest
 * scores sum to at least lambda times the total.  The scores of Eq. 6 are
 * attention masses (means of softmax probabilities, Eq. 5), so a value that is
 * not a finite positive number (negative, zero, NaN, infinite) carries no
 * mass; it keeps its place in the descending order.  The total is the last
 * prefix sum (fp64, in sorted order), so lambda = 1 is reached exactly where
 * the mass ends.  Returns c, or a negative error.  *margin (optional) receives
 * the distance of lambda*total to the nearer of the two prefix sums that
 * decide c, divided by the total. */
static double score_mass(float x)
{
    return (x > 0.0f && x < INFINITY) ? (double)x : 0.0;
}

int oracle_top_p_count(const float* scores, int n_video, double lambda, double* margin)
{
    if (n_video < 0 || !(lambda >= 0.0 && lambda <= 1.0)) return -1;
    if (margin) *margin = 1.0;
    if (n_video == 0) return 0;
    scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)n_video);
    if (!order) return -2;
    for (int j = 0; j < n_video; ++j) { order[j].key = scores[j]; order[j].idx = j; }
    qsort(order, (size_t)n_video, sizeof(scored_t), cmp_desc);
    double total = 0.0;
    for (int j = 0; j < n_video; ++j) total += score_mass(order[j].key);
    double acc = 0.0, before = 0.0;
    int c = 0;
    while (c < n_video && !(acc >= lambda * total)) { before = acc; acc += score_mass(order[c].key); ++c; }
    /* margin: how far the threshold sits from the two partial sums that decide c, relative to the total */
    if (margin && total > 0.0) {
        const double goal = lambda * total;
        const double d_hi = acc - goal;                       /* >= 0 when the loop stopped on the test */
        const double d_lo = c > 0 ? goal - before : goal;     /* > 0: the previous prefix fell short */
        *margin = (d_hi < d_lo ? d_hi : d_lo) / total;
    }
    free(order);
    return c;
}

/* ------------------------------------------------------------------------
 * Draft cache construction  (Sec. 3.2 last paragraph; Self-SD setting of
 * Sec. 4: same parameters, pruned KV cache).  Rows before the video, the kept
 * video rows in ascending order, then every row after the video (the language
 * prompt is always kept).  Pure copy of 16-bit words.
 * ---------------------------------------------------------------------- */
int oracle_gather_kv(const uint16_t* src /* [n_keys, row_elems] */, uint16_t* dst,
                     int n_keys, int video_start, int n_video,
                     const int32_t* keep_idx, int n_keep, int row_elems)
{
    if (video_start < 0 || n_video < 0 || video_start + n_video > n_keys || n_keep < 0) return -1;
    long r = 0;
    for (int j = 0; j < video_start; ++j, ++r)
        memcpy(dst + r * row_elems, src + (long)j * row_elems, sizeof(uint16_t) * (size_t)row_elems);
    for (int m = 0; m < n_keep; ++m, ++r) {
        if (keep_idx[m] < 0 || keep_idx[m] >= n_video) return -1;
        memcpy(dst + r * row_elems, src + ((long)video_start + keep_idx[m]) * row_elems,
               sizeof(uint16_t) * (size_t)row_elems);
    }
    for (int j = video_start + n_video; j < n_keys; ++j, ++r)
        memcpy(dst + r * row_elems, src + (long)j * row_elems, sizeof(uint16_t) * (size_t)row_elems);
    return 0;
}

/* ------------------------------------------------------------------------
 * Acceptance, greedy  (App. A: the target generates with greedy decoding; the
 * method is lossless, Sec. 4 Metrics).  t_i = argmax of target row i, lowest
 * index on ties; accept the longest prefix of drafted tokens with x_i == t_i,
 * then emit the target's own token at the first mismatch (or the bonus token
 * t_gamma when all match).  Unused output slots are -1.
 * ---------------------------------------------------------------------- */
static int argmax_f32(const float* x, int n)
{
    int best = 0;
    for (int v = 1; v < n; ++v) if (x[v] > x[best]) best = v;
    return best;
}

int oracle_accept_greedy(const float* target_logits /* [gamma+1, vocab] */,
                         const int32_t* draft_tokens /* [gamma] */, int gamma, int vocab,
                         int32_t* n_accepted, int32_t* out_tokens /* [gamma+1] */)
{
    if (gamma < 0 || vocab < 1) return -1;
    int n = 0;
    while (n < gamma && draft_tokens[n] == argmax_f32(target_logits + (long)n * vocab, vocab)) ++n;
    for (int i = 0; i <= gamma; ++i) out_tokens[i] = -1;
    for (int i = 0; i < n; ++i) out_tokens[i] = draft_tokens[i];
    out_tokens[n] = argmax_f32(target_logits + (long)n * vocab, vocab);
    *n_accepted = n;
    return 0;
}

/* ------------------------------------------------------------------------
 * Acceptance, rejection sampling: the rule of the speculative-sampling work
 * the paper builds on (Sec. 1 and Related Work: output distribution of the
 * target is preserved).  p_i, q_i are the softmax of target / draft row i at
 * the given temperature.
 *   for i = 0..gamma-1: accept x_i iff u_i * q_i[x_i] < p_i[x_i]; stop at the
 *   first rejection; n = number accepted.
 *   final token from w = max(p_n - q_n, 0) if n < gamma, else from p_gamma,
 *   by inverse CDF with u_gamma in ascending token order.
 * margins[i] (i < gamma) = |u_i q - p| / max(u_i q, p) of test i (or -1 if the
 * test was not reached); margins[gamma] = distance of u_gamma * W to the
 * nearest CDF step bounding the chosen token, divided by W.
 * ---------------------------------------------------------------------- */
static void softmax_f64(const float* x, int n, double inv_t, double* p)
{
    double m = -INFINITY, z = 0.0;
    for (int v = 0; v < n; ++v) { const double s = (double)x[v] * inv_t; if (s > m) m = s; }
    for (int v = 0; v < n; ++v) { p[v] = exp((double)x[v] * inv_t - m); z += p[v]; }
    for (int v = 0; v < n; ++v) p[v] /= z;
}

int oracle_accept_sample(const float* target_logits /* [gamma+1, vocab] */,
                         const float* draft_logits  /* [gamma,   vocab] */,
                         const int32_t* draft_tokens, const float* uniforms /* [gamma+1] */,
                         int gamma, int vocab, double temperature,
                         int32_t* n_accepted, int32_t* out_tokens, double* margins /* [gamma+1] or NULL */)
{
    if (gamma < 0 || vocab < 1 || !(temperature > 0.0)) return -1;
    double* p = (double*)malloc(sizeof(double) * (size_t)vocab);
    double* q = (double*)malloc(sizeof(double) * (size_t)vocab);
    double* w = (double*)malloc(sizeof(double) * (size_t)vocab);
    if (!p || !q || !w) { free(p); free(q); free(w); return -2; }
    const double inv_t = 1.0 / temperature;
    if (margins) for (int i = 0; i <= gamma; ++i) margins[i] = -1.0;
    int n = 0;
    for (; n < gamma; ++n) {
        const int x = draft_tokens[n];
        if (x < 0 || x >= vocab) { free(p); free(q); free(w); return -1; }
        softmax_f64(target_logits + (long)n * vocab, vocab, inv_t, p);
        softmax_f64(draft_logits + (long)n * vocab, vocab, inv_t, q);
        const double lhs = (double)uniforms[n] * q[x], rhs = p[x];
        if (margins) {
            const double big = lhs > rhs ? lhs : rhs;
            margins[n] = big > 0.0 ? fabs(lhs - rhs) / big : 0.0;
        }
        if (!(lhs < rhs)) break;
    }
    softmax_f64(target_logits + (long)n * vocab, vocab, inv_t, p);
    if (n < gamma) {
        softmax_f64(draft_logits + (long)n * vocab, vocab, inv_t, q);
        for (int v = 0; v < vocab; ++v) w[v] = p[v] - q[v] > 0.0 ? p[v] - q[v] : 0.0;
    } else {
        for (int v = 0; v < vocab; ++v) w[v] = p[v];
    }
    double W = 0.0;
    for (int v = 0; v < vocab; ++v) W += w[v];
    int y;
    if (!(W > 0.0)) {
        y = 0;
        for (int v = 1; v < vocab; ++v) if (p[v] > p[y]) y = v;
        if (margins) margins[gamma] = 1.0;
    } else {
        const double target = (double)uniforms[gamma] * W;
        double c = 0.0, below = 0.0;
        y = -1;
        int last_pos = 0;
        for (int v = 0; v < vocab; ++v) {
            if (w[v] > 0.0) last_pos = v;
            if (c + w[v] > target) { y = v; below = c; c += w[v]; break; }
            c += w[v];
        }
        if (y < 0) { y = last_pos; if (margins) margins[gamma] = 0.0; }
        else if (margins) {
            const double d0 = target - below, d1 = c - target;
            margins[gamma] = (d0 < d1 ? d0 : d1) / W;
        }
    }
    for (int i = 0; i <= gamma; ++i) out_tokens[i] = -1;
    for (int i = 0; i < n; ++i) out_tokens[i] = draft_tokens[i];
    out_tokens[n] = y;
    *n_accepted = n;
    free(p); free(q); free(w);
    return 0;
}

/* The final draw's distribution after n accepted drafts, as a normalised CDF
 * interval [lo, hi) of one token: lets a test check that a token returned for
 * the uniform u_gamma satisfies lo <= u_gamma < hi up to a stated slack, where
 * rounding decides between neighbouring tokens. */
int oracle_final_token_interval(const float* target_logits, const float* draft_logits,
                                int n, int gamma, int vocab, double temperature, int token,
                                double* lo, double* hi)
{
    if (n < 0 || n > gamma || vocab < 1 || token < 0 || token >= vocab || !(temperature > 0.0)) return -1;
    double* p = (double*)malloc(sizeof(double) * (size_t)vocab);
    double* q = (double*)malloc(sizeof(double) * (size_t)vocab);
    if (!p || !q) { free(p); free(q); return -2; }
    softmax_f64(target_logits + (long)n * vocab, vocab, 1.0 / temperature, p);
    if (n < gamma) {
        softmax_f64(draft_logits + (long)n * vocab, vocab, 1.0 / temperature, q);
        for (int v = 0; v < vocab; ++v) p[v] = p[v] - q[v] > 0.0 ? p[v] - q[v] : 0.0;
    }
    double W = 0.0, below = 0.0;
    for (int v = 0; v < vocab; ++v) W += p[v];
    for (int v = 0; v < token; ++v) below += p[v];
    if (!(W > 0.0)) { free(p); free(q); return -3; }
    *lo = below / W;
    *hi = (below + p[token]) / W;
    free(p); free(q);
    return 0;
}

/* ------------------------------------------------------------------------
 * Tree-masked verification  (Sec. 3.2 "Bonus": the draft tree is verified in
 * one target forward through a specialised attention mask; App. B).
 * The block's q_len tokens are tree nodes; node t sees every key before the
 * block and, inside the block, node b iff bit b of mask[t] is set (its
 * ancestors and itself).  A chain's mask, bits 0..t, gives oracle_decode_attn.
 * ---------------------------------------------------------------------- */
int oracle_tree_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint64_t* mask,
                     int q_len, int kv_len, int n_q_heads, int n_kv_heads, int d,
                     double scale, double* out, double* lse)
{
    if (q_len < 0 || q_len > 64 || kv_len < q_len || n_kv_heads < 1 || n_q_heads % n_kv_heads) return -1;
    const int group = n_q_heads / n_kv_heads, ctx = kv_len - q_len;
    const long rows = (long)q_len * n_q_heads;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        const int t = (int)(r / n_q_heads), h = (int)(r % n_q_heads), g = h / group;
        const uint16_t* qv = q + ((long)t * n_q_heads + h) * d;
        double* s = (double*)malloc(sizeof(double) * (size_t)(kv_len > 0 ? kv_len : 1));
        if (!s) { failed = 1; continue; }
        double m = -INFINITY, z = 0.0;
        for (int j = 0; j < kv_len; ++j) {
            const int seen = j < ctx || ((mask[t] >> (j - ctx)) & 1);
            s[j] = seen ? scale * dot_bf16(qv, k + ((long)j * n_kv_heads + g) * d, d) : -INFINITY;
            if (s[j] > m) m = s[j];
        }
        for (int j = 0; j < kv_len; ++j) if (s[j] > -INFINITY) z += exp(s[j] - m);
        double* o = out + r * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j < kv_len; ++j) {
            if (!(s[j] > -INFINITY)) continue;
            const double p = exp(s[j] - m) / z;
            const uint16_t* vv = v + ((long)j * n_kv_heads + g) * d;
            for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f64(vv[c]);
        }
        if (lse) lse[r] = m + log(z);
        free(s);
    }
    return failed ? -2 : 0;
}

/* ------------------------------------------------------------------------
 * Greedy acceptance over a draft tree  (App. B: verifying several candidates in
 * one forward raises the accept length).  Node 0 is the last committed token;
 * parent[i] < i for i >= 1.  Starting at node 0: the target's token at the
 * current node is the argmax of its row (lowest index on ties); move to the
 * lowest-numbered child that drafted exactly that token, if any.  The emitted
 * tokens are the accepted nodes' tokens followed by the target's token at the
 * node where the walk stops -- the target's own greedy continuation.
 * ---------------------------------------------------------------------- */
int oracle_accept_tree_greedy(const float* target_logits /* [n_nodes, vocab] */,
                              const int32_t* node_tokens /* [n_nodes], entry 0 unused */,
                              const int32_t* parent /* [n_nodes], parent[0] = -1 */,
                              int n_nodes, int vocab, int32_t* n_accepted,
                              int32_t* accepted_nodes /* [n_nodes] */, int32_t* out_tokens /* [n_nodes] */)
{
    if (n_nodes < 1 || vocab < 1) return -1;
    for (int i = 1; i < n_nodes; ++i) if (parent[i] < 0 || parent[i] >= i) return -1;
    for (int i = 0; i < n_nodes; ++i) { accepted_nodes[i] = -1; out_tokens[i] = -1; }
    int cur = 0, n = 0;
    for (;;) {
        const int t = argmax_f32(target_logits + (long)cur * vocab, vocab);
        int next = -1;
        for (int c = cur + 1; c < n_nodes && next < 0; ++c)
            if (parent[c] == cur && node_tokens[c] == t) next = c;
        if (next < 0) { out_tokens[n] = t; break; }
        accepted_nodes[n] = next;
        out_tokens[n] = node_tokens[next];
        ++n;
        cur = next;
    }
    *n_accepted = n;
    return 0;
}

/* ------------------------------------------------------------------------
 * Attention-agnostic retention sets the paper compares against (Sec. 5.2 ablation
 * and "Exploration of Diverse Pruning Criteria"; the random pruning of Sec. 2.2).
 * Video tokens are numbered frame-major, then row-major on the frame's
 * grid_h x grid_w grid.  Every mode writes ascending indices and returns how
 * many it wrote (negative: invalid arguments).
 *   0 window, front  : tokens 0 .. B-1
 *   1 window, middle : B consecutive tokens starting at floor((V-B)/2)
 *   2 window, end    : tokens V-B .. V-1
 *   3 uniform, flat  : tokens floor(t*V/B), t = 0..B-1 (Stage II alone, nothing taken by Stage I)
 *   4 frame dropping : F_k = floor(B / tokens per frame) whole frames at the regular
 *                      temporal interval F/F_k: frames floor(t*F/F_k)
 *   5 spatial lattice: in every frame the grid positions whose row is a multiple of
 *                      stride_h and whose column is a multiple of stride_w (B unused)
 *   6 random         : token j draws the 30 high bits of the j-th output of the
 *                      SplitMix64 generator seeded with `seed`; the B largest draws
 *                      are kept (equal draws: lower index first)
 * ---------------------------------------------------------------------- */
uint64_t oracle_splitmix64(uint64_t seed, uint64_t j)   /* j-th output (j = 0 first) of the stream */
{
    uint64_t z = seed + (j + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

typedef struct { uint32_t draw; int32_t idx; } drawn_t;

static int cmp_draw_desc(const void* pa, const void* pb)
{
    const drawn_t* a = (const drawn_t*)pa;
    const drawn_t* b = (const drawn_t*)pb;
    if (a->draw != b->draw) return a->draw > b->draw ? -1 : 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

static int cmp_i32(const void* pa, const void* pb)
{
    const int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
    return (a > b) - (a < b);
}

int oracle_baseline_keep(int mode, int n_video, int n_frames, int grid_h, int grid_w,
                         int keep_budget, int stride_h, int stride_w, uint64_t seed,
                         int32_t* keep_idx)
{
    const int64_t V = n_video, B = keep_budget;
    if (V < 0 || B < 0 || B > V) return -1;
    const int64_t tpf = (int64_t)grid_h * grid_w;
    if (mode == 4 || mode == 5 || mode == 7) {
        if (n_frames < 0 || grid_h <= 0 || grid_w <= 0 || tpf * n_frames != V) return -1;
    }
    int n = 0;
    switch (mode) {
    case 0: for (int64_t t = 0; t < B; ++t) keep_idx[n++] = (int32_t)t; break;
    case 1: for (int64_t t = 0; t < B; ++t) keep_idx[n++] = (int32_t)((V - B) / 2 + t); break;
    case 2: for (int64_t t = 0; t < B; ++t) keep_idx[n++] = (int32_t)(V - B + t); break;
    case 3: for (int64_t t = 0; t < B; ++t) keep_idx[n++] = (int32_t)((t * V) / B); break;
    case 4: {
        const int64_t fk = B / tpf;
        for (int64_t t = 0; t < fk; ++t) {
            const int64_t f = (t * n_frames) / fk;
            for (int64_t w = 0; w < tpf; ++w) keep_idx[n++] = (int32_t)(f * tpf + w);
        }
        break;
    }
    case 5:
        if (stride_h <= 0 || stride_w <= 0) return -1;
        for (int f = 0; f < n_frames; ++f)
            for (int r = 0; r < grid_h; r += stride_h)
                for (int c = 0; c < grid_w; c += stride_w)
                    keep_idx[n++] = (int32_t)(f * tpf + (int64_t)r * grid_w + c);
        break;
    case 6: {
        drawn_t* order = (drawn_t*)malloc(sizeof(drawn_t) * (size_t)(V > 0 ? V : 1));
        if (!order) return -2;
        for (int64_t j = 0; j < V; ++j) {
            order[j].draw = (uint32_t)(oracle_splitmix64(seed, (uint64_t)j) >> 34);
            order[j].idx = (int32_t)j;
        }
        qsort(order, (size_t)V, sizeof(drawn_t), cmp_draw_desc);
        for (int64_t t = 0; t < B; ++t) keep_idx[n++] = order[t].idx;
        qsort(keep_idx, (size_t)n, sizeof(int32_t), cmp_i32);
        free(order);
        break;
    }
    case 7:
        /* Eq. 7 with an empty V_R, restarted in every frame: the budget is dealt to the frames in
         * order (frame f gets the output positions floor(f*B/F) .. floor((f+1)*B/F) - 1) and each
         * frame strides its own grid from its first token. */
        for (int64_t f = 0; f < n_frames; ++f) {
            const int64_t lo = (f * B) / n_frames, hi = ((f + 1) * B) / n_frames;
            for (int64_t u = 0; u < hi - lo; ++u)
                keep_idx[n++] = (int32_t)(f * tpf + (u * tpf) / (hi - lo));
        }
        break;
    default: return -1;
    }
    return n;
}
