/*
 * specvlm.h -- C ABI of the SpecVLM speculative-decode hot path on MI355X.
 *
 * One operation per step of a speculative decode step of a video LLM over a
 * long video KV cache (paper: arXiv 2508.16201), and the variants of them the
 * paper's tree decoding and ablations need:
 *
 *   specvlm_score        language-to-video attention scores   (Sec. 3.1, Eq. 4-5)
 *   specvlm_score_layers the same, summed over all layers in one call
 *   specvlm_select       Stage I top-k + Stage II uniform stride (Sec. 3.2, Eq. 6-7)
 *   specvlm_top_p_count  Stage I's size by cumulative score mass (Sec. 3.2, Eq. 6)
 *   specvlm_gather_kv    the draft's pruned KV cache           (Sec. 3.2, last paragraph)
 *   specvlm_decode_attn  draft decode / parallel verification  (Sec. 2.1)
 *   specvlm_accept       draft-token acceptance                (Sec. 2.1; App. A greedy)
 *   specvlm_tree_attn / specvlm_accept_tree   the same two steps for a draft tree (App. B)
 *   specvlm_baseline_keep  retention sets of the attention-agnostic pruners (Sec. 2.2, 5.2)
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Return value: SPECVLM_OK (0) or a negative SPECVLM_E* code.  Arguments are
 *    validated on the host before anything is enqueued: a failed call has
 *    launched nothing.  Nothing is printed, nothing aborts.
 *  - Every data pointer is a DEVICE pointer owned by the caller unless it is
 *    marked "host".  The library never allocates, frees or keeps a pointer.
 *    Scratch memory comes from the caller as `workspace` (device, 256-byte
 *    aligned); its required size is returned by the matching
 *    specvlm_*_workspace_bytes query, which is host-only and pure.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work and return without synchronising; outputs are valid
 *    once the stream reaches that point.  Calls that share a workspace must be
 *    ordered on one stream.
 *  - bf16 tensors are described by (pointer, token stride, head stride) in
 *    ELEMENTS; the head dimension d is contiguous and rows are 16-byte aligned
 *    (strides are multiples of 8 elements).  Both [tokens, heads, d] and
 *    [heads, tokens, d] caches are therefore accepted without a copy.
 *  - Supported shapes: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads;
 *    anything else returns SPECVLM_EUNSUPPORTED.
 *  - Ragged batches: `cu_*` are device int32 arrays of batch+1 prefix offsets
 *    (request b owns rows [cu[b], cu[b+1]) of the concatenated tensor).  A NULL
 *    cu pointer means batch = 1 with the scalar length arguments.  With cu
 *    arrays the scalar length arguments are the MAXIMUM over requests (they
 *    size the launch); the device arrays are trusted to respect them.
 *  - Zero-size work (batch 0, no video tokens, budget 0) is legal: returns 0.
 */
#ifndef SPECVLM_H
#define SPECVLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPECVLM_OK            0
#define SPECVLM_EINVAL       (-1)  /* invalid argument (null pointer, negative size, budget > tokens, ...) */
#define SPECVLM_EUNSUPPORTED (-2)  /* shape outside the supported set */
#define SPECVLM_EWORKSPACE   (-3)  /* workspace missing, misaligned or too small */
#define SPECVLM_ELAUNCH      (-4)  /* the HIP runtime refused a launch */

/* Static text for a return code (host pointer, never NULL). */
const char* specvlm_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int specvlm_version(void);

/* --------------------------------------------------------------------------
 * specvlm_score -- token scores A = {a_j}  (Sec. 3.1, Eq. 4-5).
 *
 * The guidance matrix G is the language-query x video-key block of the
 * verifier's attention matrix; a_j is column j of G averaged over the language
 * queries (Eq. 5) and over the q heads of this layer (Sec. 3.1 takes the mean
 * over the layers as well: layers are accumulated by calling once per layer
 * with beta = 1, or all at once by specvlm_score_layers).
 *
 *   q_text   bf16 [n_text, H_q, d]   language-prompt queries (RoPE already applied)
 *   k_cache  bf16 [n_keys, H_kv, d]  this layer's keys
 *   video keys are rows [video_start, video_start + n_video) of k_cache
 *   text query i sits at absolute position text_pos0 + i and sees keys
 *   j <= text_pos0 + i (causal); softmax logits are softmax_scale * q.k
 *   norm_mode 0: rows normalised over every visible key, then sliced to the
 *                video columns (G is a block of the full attention matrix)
 *   norm_mode 1: rows normalised over the visible video keys only
 *   row_lse  optional fp32 [n_text, H_q]: natural-log normaliser of each row for
 *            the chosen norm_mode (e.g. saved by the prefill attention); when
 *            given, the library skips its own normaliser pass
 *   scores   fp32 [n_video]:  scores = beta * scores + (1/(H_q n_text)) sum_{h,i} G
 *            (beta = 0 overwrites and never reads the old contents)
 *
 * A batch (one set of launches for all requests): the requests are
 * concatenated along the token axis of q_text, k_cache, row_lse and scores, and
 * cu_text, cu_keys, cu_video are DEVICE int32 arrays of batch+1 prefix offsets,
 * as in every other call.  n_text, n_keys, n_video are then the maxima over the
 * batch (host ints: they size the launches and the workspace; the split plan is
 * made from them and a request's workgroups find their real sizes on the
 * device); video_start applies inside every request; text_pos0 = -1 places each
 * request's text queries on its last n_text_b keys (text_pos0 >= 0 is the same
 * position for every request).  A request whose device-side sizes exceed the
 * maxima or do not fit together (video_start + n_video_b > n_keys_b) is skipped:
 * its scores are left untouched.  With all three NULL, batch must be 1 and
 * text_pos0 = -1 means n_keys - n_text.
 * The workspace query takes the batch and the same maxima.
 * -------------------------------------------------------------------------- */
size_t specvlm_score_workspace_bytes(int batch, int n_text, int n_keys, int n_video,
                                     int n_q_heads, int n_kv_heads, int head_dim,
                                     int have_row_lse);

int specvlm_score(
    const void* q_text,  int64_t q_tok_stride, int64_t q_head_stride,
    const void* k_cache, int64_t k_tok_stride, int64_t k_head_stride,
    const int32_t* cu_text, const int32_t* cu_keys, const int32_t* cu_video, int batch,
    int n_text, int n_keys, int video_start, int n_video, int text_pos0,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    int norm_mode, const float* row_lse, float beta, float* scores,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_score_layers -- the same scores, summed over n_layers layers in one
 * call (Sec. 3.1 takes the importance as a mean over the verifier's layers as
 * well as its heads; the sum over layers is what n_layers calls of
 * specvlm_score with beta = 1 accumulate):
 *
 *   scores = beta * scores + sum_l (1/(H_q n_text)) sum_{h,i} G_l
 *
 * Layer l reads q_text + l * q_layer_stride and k_cache + l * k_layer_stride
 * (strides in elements, multiples of 8; 0 is allowed and reads the same tensor
 * again) and, when row_lse is given, row_lse + l * row_lse_layer_stride floats.
 * Everything else is as for specvlm_score, including the batch.  One set of four
 * launches serves all layers (a caller that keeps the text queries of every
 * layer until the prefill has ended pays for 4 launches instead of 4 n_layers,
 * and every launch has n_layers times the workgroups to fill the chip with).
 * n_layers = 0 only applies beta.  n_layers * batch <= 65535.
 * The workspace query takes n_layers as well; the result is deterministic (the
 * layers are added in the order 0, 1, ...), and equals what the per-layer calls
 * give up to the rounding of one fp32 sum taken in a different order.
 * -------------------------------------------------------------------------- */
size_t specvlm_score_layers_workspace_bytes(int n_layers, int batch, int n_text, int n_keys, int n_video,
                                            int n_q_heads, int n_kv_heads, int head_dim,
                                            int have_row_lse);

int specvlm_score_layers(
    const void* q_text,  int64_t q_layer_stride, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k_cache, int64_t k_layer_stride, int64_t k_tok_stride, int64_t k_head_stride, int n_layers,
    const int32_t* cu_text, const int32_t* cu_keys, const int32_t* cu_video, int batch,
    int n_text, int n_keys, int video_start, int n_video, int text_pos0,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    int norm_mode, const float* row_lse, int64_t row_lse_layer_stride, float beta, float* scores,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_select -- the two-stage retention set  (Sec. 3.2).
 *
 * Stage I: V_R = the k_top highest-scoring video tokens (Eq. 6 sizes V_R by
 *   cumulative score mass; here its size is an input).  Equal scores: the
 *   lower token index ranks first.
 *   -0.0 equals +0.0; NaN ranks below every number.
 * Stage II: over the remaining tokens V \ V_R in raster order (frame-major,
 *   row-major inside a frame), keep U = keep_budget - k_top tokens at the fixed
 *   interval I = R/U (Eq. 7 with the budget as denominator), R = n_video - k_top:
 *   the tokens whose rank in the remainder is floor(t*R/U), t = 0..U-1.
 * Output: keep_idx = sort(V_R u V_U), ascending, video-local, exactly
 *   keep_budget entries per request; from_topk[m] = 1 iff keep_idx[m] is in V_R.
 *
 *   scores      fp32 [sum n_video_b]
 *   cu_video    int32 [batch+1] or NULL (batch 1, n_video = max_n_video)
 *   k_top, keep_budget   device int32 [batch]
 *   cu_keep     device int32 [batch+1], prefix sums of keep_budget; NULL for batch 1
 *   max_n_video, total_keep   host ints (launch shape, validation)
 *   keep_idx    int32 [total_keep];  from_topk  uint8 [total_keep] or NULL
 *   status      optional device int32 [batch]: SPECVLM_OK, or SPECVLM_EINVAL for a
 *               request whose device-side budgets are inconsistent (k_top >
 *               keep_budget, keep_budget > n_video, n_video > max_n_video); such
 *               a request writes no indices.
 * Limit: max_n_video <= 65536.  No workspace is needed (the query returns 0).
 * -------------------------------------------------------------------------- */
size_t specvlm_select_workspace_bytes(int batch, int max_n_video);

int specvlm_select(
    const float* scores, const int32_t* cu_video,
    const int32_t* k_top, const int32_t* keep_budget, const int32_t* cu_keep,
    int batch, int max_n_video, int total_keep,
    int32_t* keep_idx, uint8_t* from_topk, int32_t* status,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_top_p_count -- Stage I's own size rule  (Sec. 3.2, Eq. 6): for each
 * request, count[b] = the smallest c such that the c largest scores sum to at
 * least lambda times the sum of all scores (0 when the total is 0 or lambda
 * is 0), clamped to max_count[b] when max_count is given.  The result can be
 * passed to specvlm_select as k_top (with max_count = keep_budget).
 * Scores are attention masses: a value that is not a finite positive number
 * (negative, zero, NaN, infinite) adds no mass and keeps its place in the
 * descending order.  Sums are exact 64-bit fixed point (2^-40 of the largest score), so the
 * result is deterministic; it can differ from an fp64 evaluation only when
 * lambda * total lies within ~1e-9 * total of a prefix sum.
 *   scores fp32 [sum n_video_b]; cu_video int32 [batch+1] or NULL (batch 1);
 *   max_count device int32 [batch] or NULL; count device int32 [batch].
 * Limit: max_n_video <= 65536.  No workspace is needed (the query returns 0).
 * -------------------------------------------------------------------------- */
size_t specvlm_top_p_count_workspace_bytes(int batch, int max_n_video);

int specvlm_top_p_count(
    const float* scores, const int32_t* cu_video, int batch, int max_n_video,
    float lambda, const int32_t* max_count, int32_t* count,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_gather_kv -- build the draft's KV cache  (Sec. 3.2, last paragraph:
 * the draft keeps V_R u V_U and the language prompt; Self-SD setting: same
 * parameters, pruned KV cache).  For every layer, for K and V:
 *
 *   dst rows = src[0 : video_start]  ++  src[video_start + keep_idx[*]]
 *              ++  src[video_start + n_video : n_keys]
 *
 * Rows are copied bit for bit.  src/dst: bf16 [n_layers, tokens, H_kv, d] with
 * explicit layer / token / head strides (elements).  dst holds
 * n_keys - n_video + n_keep tokens per layer.  keep_idx is device int32
 * [n_keep], video-local, ascending (the output of specvlm_select).  dst must
 * not overlap src.  v_src/v_dst may both be NULL to copy K only.
 *
 * A batch (one launch for all requests): the requests are concatenated along
 * the token axis of src, dst and keep_idx; cu_keys, cu_video, cu_keep are
 * device int32 [batch+1] prefix offsets of the requests' source rows, video
 * tokens and kept tokens (cu_video and cu_keep are the arrays specvlm_select
 * takes), and n_keys, n_video, n_keep are the TOTALS over the batch (host
 * ints: they size the launch).  Request b's destination rows start at
 * cu_keys[b] - cu_video[b] + cu_keep[b]; video_start applies inside every
 * request.  All three NULL: one request (batch must be 0 or 1).
 *
 *   status  optional device int32 [1]: SPECVLM_OK, or SPECVLM_EINVAL when some
 *           keep_idx entry lies outside its request's video span or a request's
 *           device-side sizes do not fit together (n_keep_b > n_video_b,
 *           video_start + n_video_b > n_keys_b).  A destination row without a
 *           valid source is zero-filled; nothing is read out of bounds.  With
 *           status NULL the same rows are zero-filled silently.
 * -------------------------------------------------------------------------- */
int specvlm_gather_kv(
    const void* k_src, const void* v_src,
    int64_t src_layer_stride, int64_t src_tok_stride, int64_t src_head_stride,
    void* k_dst, void* v_dst,
    int64_t dst_layer_stride, int64_t dst_tok_stride, int64_t dst_head_stride,
    int n_layers, int n_keys, int video_start, int n_video,
    const int32_t* keep_idx, int n_keep,
    const int32_t* cu_keys, const int32_t* cu_video, const int32_t* cu_keep, int batch,
    int32_t* status, int n_kv_heads, int head_dim, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_decode_attn -- grouped-query softmax attention of a short query
 * block over a KV cache  (Sec. 2.1).  q_len = 1 is the draft's (or target's)
 * plain decode; q_len = gamma + 1 is the target's parallel verification of
 * gamma drafted tokens: the block is the last committed token followed by the
 * drafted ones, its own K/V rows are already the last q_len rows of the cache,
 * and request-local key j is visible to query t iff j <= kv_len - q_len + t
 * (causal inside the block).
 *
 *   q    bf16 [sum q_len_b, H_q, d]      out  bf16, same shape and strides as q
 *   k,v  bf16 [sum kv_len_b, H_kv, d]    (one token / head stride pair for both)
 *   lse  optional fp32 [sum q_len_b, H_q]: natural log of each row's softmax sum
 *   q head h reads kv head h / (H_q / H_kv)
 *   num_splits: key-range splits per (request, kv head) (flash-decode);
 *               0 lets the library choose for the shape.  For a batch of 2..64
 *               requests the choice is made on the device from the request
 *               lengths: the key tiles of the requests are dealt in equal
 *               contiguous runs to groups of n_kv_heads workgroups (one per
 *               head, one workgroup per CU), so requests of very different
 *               lengths finish together.
 *   Workspace: the query takes the same batch, maxima, head counts and
 *               num_splits as the call (it is pure: it depends on nothing else).
 * Limits: q_len <= 64.  Up to 64 query rows per kv head ((H_q/H_kv) * q_len)
 *   read K and V from memory exactly once; beyond that the rows are processed in
 *   groups of at most 64 (one workgroup per group, head and key range) and each
 *   group reads the key range again, its neighbours' copy mostly still cached.
 * -------------------------------------------------------------------------- */
size_t specvlm_decode_attn_workspace_bytes(int batch, int q_len, int kv_len,
                                           int n_q_heads, int n_kv_heads, int head_dim,
                                           int num_splits);

int specvlm_decode_attn(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    void* out, float* lse, int num_splits,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_decode_attn_static -- specvlm_decode_attn for callers that cannot
 * allocate device memory or hand over a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as specvlm_decode_attn without the workspace pair; the
 * split-K partial results live in an array inside the library's device image
 * (specvlm_decode_attn_static_scratch_bytes() = 16 MiB, held by every GPU that
 * loads the library until the process ends).  The call allocates nothing and
 * frees nothing.
 *   - A shape whose specvlm_decode_attn_workspace_bytes exceeds that size
 *     returns SPECVLM_EWORKSPACE and launches nothing.
 *   - All calls on one GPU share the array: calls must be ordered on one
 *     stream (or otherwise not overlap); overlapping calls race.  The array
 *     keeps the previous call's contents; the kernels never read a slot they
 *     have not written in the same call.
 * -------------------------------------------------------------------------- */
size_t specvlm_decode_attn_static_scratch_bytes(void);

int specvlm_decode_attn_static(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    void* out, float* lse, int num_splits, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_tree_attn -- specvlm_decode_attn for a block of draft-TREE nodes
 * (Sec. 3.2 "Bonus" and App. B: the tree is verified in one target forward
 * through a specialised attention mask).  Same arguments as specvlm_decode_attn
 * plus
 *   ancestor_mask  device uint64 [sum q_len_b]: query t of a request sees every
 *                  key before its block and block key b iff bit b of its mask
 *                  is set (node b is t itself or one of its ancestors).  Every
 *                  row must have its own bit set.  q_len <= 64.
 * The chain mask (bits 0..t for query t) reproduces specvlm_decode_attn.
 * Workspace: specvlm_decode_attn_workspace_bytes of the same shape.
 * -------------------------------------------------------------------------- */
int specvlm_tree_attn(
    const void* q, int64_t q_tok_stride, int64_t q_head_stride,
    const void* k, const void* v, int64_t kv_tok_stride, int64_t kv_head_stride,
    const int32_t* cu_q, const int32_t* cu_kv, int batch, int q_len, int kv_len,
    int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale,
    const uint64_t* ancestor_mask, void* out, float* lse, int num_splits,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_accept -- which drafted tokens survive verification  (Sec. 2.1).
 *
 * Greedy (uniforms == NULL, then draft_logits must be NULL too; App. A: the target decodes
 * greedily, output identical to the target's own): t_i = argmax of target row
 * i, lowest index on ties; n = length of the longest prefix with
 * draft_tokens[i] == t_i; out = x_0..x_{n-1}, t_n, then -1 padding.
 *
 * Rejection sampling (uniforms given, draft_logits required when gamma > 0; the speculative-sampling rule the paper
 * builds on, which preserves the target's output distribution): with p_i, q_i
 * the softmax of target / draft row i at `temperature`, accept x_i iff
 * u_i * q_i[x_i] < p_i[x_i], stop at the first rejection (n accepted); the
 * final token is drawn by inverse CDF (ascending token order) with u_gamma from
 * max(p_n - q_n, 0) if n < gamma, else from p_gamma.
 *
 *   target_logits fp32 [batch, gamma+1, vocab]   draft_logits fp32 [batch, gamma, vocab]
 *   draft_tokens  int32 [batch, gamma]           uniforms     fp32 [batch, gamma+1] in [0,1)
 *   n_accepted    int32 [batch] (0..gamma)       out_tokens   int32 [batch, gamma+1]
 * -------------------------------------------------------------------------- */
size_t specvlm_accept_workspace_bytes(int batch, int gamma, int vocab, int sampling);

int specvlm_accept(
    const float* target_logits, const float* draft_logits,
    const int32_t* draft_tokens, const float* uniforms,
    int batch, int gamma, int vocab, float temperature,
    int32_t* n_accepted, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_accept_tree -- greedy acceptance over a static draft tree (App. B).
 * Row i of target_logits is the target's next-token distribution at tree node
 * i; node 0 is the last committed token, parent[i] < i for i >= 1 (one tree
 * shared by the batch).  Starting at node 0: t = argmax of the current node's
 * row (lowest index on ties); move to the lowest-numbered child whose drafted
 * token equals t; stop when there is none.
 *   target_logits fp32 [batch, n_nodes, vocab]   node_tokens int32 [batch, n_nodes] (entry 0 unused)
 *   parent int32 [n_nodes] (device)              n_accepted int32 [batch]
 *   accepted_nodes int32 [batch, n_nodes]: the accepted path, then -1
 *   out_tokens int32 [batch, n_nodes]: the accepted tokens, the target's token at
 *               the stopping node, then -1 (the target's own greedy continuation)
 * n_nodes <= 64.
 * -------------------------------------------------------------------------- */
size_t specvlm_accept_tree_workspace_bytes(int batch, int n_nodes, int vocab);

int specvlm_accept_tree(
    const float* target_logits, const int32_t* node_tokens, const int32_t* parent,
    int batch, int n_nodes, int vocab,
    int32_t* n_accepted, int32_t* accepted_nodes, int32_t* out_tokens,
    void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_baseline_keep -- retention sets of the attention-agnostic pruners the
 * ablations compare with (Sec. 2.2 random pruning; Sec. 5.2: windows over the
 * front / middle / end of the video, SD-Uniform, SD-Frame).  One request.
 * Video tokens are numbered frame-major, then row-major on the frame's
 * grid_h x grid_w grid; V = n_video, B = keep_budget (0 <= B <= V).
 *   WINDOW_FRONT   tokens 0..B-1
 *   WINDOW_MIDDLE  B consecutive tokens from floor((V-B)/2)
 *   WINDOW_END     tokens V-B..V-1
 *   UNIFORM        tokens floor(t*V/B), t = 0..B-1 (Eq. 7 with an empty V_R)
 *   FRAME_DROP     F_k = floor(B / (grid_h*grid_w)) whole frames, frames floor(t*F/F_k)
 *   LATTICE        in every frame the rows that are multiples of stride_h and the
 *                  columns that are multiples of stride_w (B unused)
 *   UNIFORM_PER_FRAME  the uniform stride restarted in every frame: frame f owns the
 *                  output positions floor(f*B/F) .. floor((f+1)*B/F) - 1 (B_f of them)
 *                  and keeps its tokens floor(u*grid_h*grid_w/B_f), u = 0..B_f-1
 *   RANDOM         token j draws the 30 high bits of output j of the SplitMix64
 *                  stream seeded with `seed`; the B largest draws are kept, equal
 *                  draws by lower index (V <= 65536)
 * FRAME_DROP, LATTICE and UNIFORM_PER_FRAME need n_frames*grid_h*grid_w == V; the other modes
 * ignore the grid arguments.  specvlm_baseline_count (host arithmetic only)
 * returns how many indices the mode writes, or a negative status;
 * keep_idx (device int32, that many entries) receives them in ascending order.
 * Only RANDOM needs a workspace.
 * -------------------------------------------------------------------------- */
#define SPECVLM_BASELINE_WINDOW_FRONT  0
#define SPECVLM_BASELINE_WINDOW_MIDDLE 1
#define SPECVLM_BASELINE_WINDOW_END    2
#define SPECVLM_BASELINE_UNIFORM       3
#define SPECVLM_BASELINE_FRAME_DROP    4
#define SPECVLM_BASELINE_LATTICE       5
#define SPECVLM_BASELINE_RANDOM        6
#define SPECVLM_BASELINE_UNIFORM_PER_FRAME 7

int specvlm_baseline_count(int mode, int n_video, int n_frames, int grid_h, int grid_w,
                           int keep_budget, int stride_h, int stride_w);

size_t specvlm_baseline_workspace_bytes(int mode, int n_video);

int specvlm_baseline_keep(
    int mode, int n_video, int n_frames, int grid_h, int grid_w,
    int keep_budget, int stride_h, int stride_w, uint64_t seed,
    int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * specvlm_probe_read -- diagnostic, not a step of the method: one launch that
 * merely reads `bytes_a` bytes at `a` and `bytes_b` bytes at `b` (device
 * pointers, 16-byte aligned, sizes multiples of 16; either may be empty) with
 * 2048 workgroups of plain 16-byte loads.  The benchmark times it over a
 * layer's K and V to print what a bare read of the same bytes costs on the
 * machine at hand, beside the attention kernel's time (Sec. 2.1: decoding is
 * bound by moving the KV cache).  `sink` (device, 4 bytes, may be NULL) is
 * never written in practice.
 * -------------------------------------------------------------------------- */
int specvlm_probe_read(const void* a, size_t bytes_a, const void* b, size_t bytes_b,
                       void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVLM_H */
