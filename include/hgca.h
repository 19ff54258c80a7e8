/*
 * libhgca -- decode-time hybrid attention of HGCA (arXiv 2507.03153) for one
 * AMD MI355X (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * The paper (Sec. 3.3, Alg. 2) computes one decode step of an attention layer
 * in two coordinated parts and a lossless aggregation:
 *   1. dense attention of the new query over the W most recent KV entries,
 *      returning the partial output O and its log-sum-exp;
 *   2. per-head sparse attention over the salient entries selected from the
 *      older, offloaded context, returning O and lse likewise;
 *   3. merge_state: O = (e^{lse_c} O_c + e^{lse_g} O_g) / (e^{lse_c} + e^{lse_g}).
 * Selection of the salient entries (Sec. 3.2.2) is per head.  In the paper the
 * older context lives in host memory and part 2 runs on CPU cores; here both
 * tiers are HBM buffers on the same GPU and all parts are GPU kernels.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - `hgca_shape` and `hgca_kv_view` structs are HOST memory, read during the
 *    call only.  Every other pointer is DEVICE memory owned by the caller.
 *    The library never allocates, frees or synchronises: a call validates its
 *    arguments on the host, enqueues kernels on `hip_stream` (a hipStream_t
 *    passed as void*, NULL = the default stream) and returns.
 *  - q is [B, Hq, d] in `shape.dtype` (fp32, or bf16 as 16-bit patterns).
 *    Query head h reads KV head h / (Hq / Hkv).
 *  - A KV tier (`hgca_kv_view`) is contiguous, k/v = [B, Hkv, cap, d], or paged,
 *    k/v = [n_blocks, Hkv, block_size, d] with logical token t of sequence b in
 *    physical block block_table[b * max_blocks + first_block[b] + t / block_size]
 *    (first_block = NULL counts as 0), slot t % block_size; the caller guarantees
 *    that the entries a sequence's valid tokens reach lie inside its table row.
 *    Two tiers may share one table: the window and the older pool of a sequence
 *    are then two ranges of the same list of blocks (see hgca_cache_state).
 *    Valid tokens of sequence b are [0, seq_lens[b]) (all `cap` when seq_lens is
 *    NULL).  The order of tokens inside a tier does not matter to the result
 *    (softmax attention is a function of the key set).  A tier holds fewer than
 *    2^32 rows (B*Hkv*cap, or n_blocks*Hkv*block_size).
 *  - Scores are s_j = sm_scale * <q, k_j>; lse is the natural log of sum e^{s_j}.
 *  - Partial outputs are fp32: O [B, Hq, d], lse [B, Hq].  An empty set gives
 *    O = 0 and lse = -inf.
 *  - q, k, v and O pointers must be 16-byte aligned.  head_dim is 64 or 128;
 *    batch and n_q_heads are at most 65 535 each.
 *  - `ws` is scratch the caller provides (split partials, score lists,
 *    histograms); its required size for a call is `hgca_workspace_bytes` with
 *    the maxima of that call.  Its contents are undefined between calls; two
 *    calls that run concurrently (different streams) need different `ws`.
 *  - Return value: HGCA_OK, or a negative hgca_status for errors the host can
 *    see (bad arguments, unsupported shape, short workspace, launch failure).
 *    On error nothing has been enqueued.  batch == 0 is a valid no-op.
 */
#ifndef HGCA_H
#define HGCA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HGCA_OK = 0,
    HGCA_ERR_INVALID_ARG = -1,   /* null/misaligned pointer, negative size, k > k_max ... */
    HGCA_ERR_UNSUPPORTED = -2,   /* head_dim, dtype, group size or block size not built */
    HGCA_ERR_WORKSPACE = -3,     /* ws is NULL or smaller than hgca_workspace_bytes()     */
    HGCA_ERR_DEVICE = -4         /* the HIP runtime refused a launch                      */
} hgca_status;

typedef enum { HGCA_F32 = 0, HGCA_BF16 = 1 } hgca_dtype;

typedef struct {
    int32_t dtype;        /* hgca_dtype of q, K and V                 */
    int32_t batch;        /* B                                        */
    int32_t n_q_heads;    /* Hq                                       */
    int32_t n_kv_heads;   /* Hkv, divides Hq; Hq/Hkv in {1,2,4,8}     */
    int32_t head_dim;     /* d, 64 or 128                             */
    float   sm_scale;     /* multiplies <q,k>; typically 1/sqrt(d)    */
} hgca_shape;

typedef struct {
    const void    *k, *v;         /* device; v may be NULL where only keys are read   */
    const int32_t *seq_lens;      /* device [B] or NULL                                */
    const int32_t *block_table;   /* device [B, max_blocks] or NULL (= contiguous)     */
    int32_t cap;                  /* capacity in tokens per sequence (logical)         */
    int32_t block_size;           /* paged only: tokens per block, a multiple of 16    */
    int32_t max_blocks;           /* paged only: row length of block_table             */
    const int32_t *first_block;   /* paged only, device [B] or NULL (= 0): the tier    */
                                  /* starts at entry first_block[b] of its table row   */
} hgca_kv_view;

/* Text for a status code (static storage). */
const char *hgca_status_string(int status);

/* Bytes of `ws` sufficient for any of the calls below on `shape` with a window
 * of at most max_window tokens, a pool of at most max_pool tokens and at most
 * k_max selected entries per head.  Returns 0 if the shape is invalid. */
size_t hgca_workspace_bytes(const hgca_shape *shape, int32_t max_window,
                            int32_t max_pool, int32_t k_max);

/* GPU-local dense attention (Sec. 3.3 "GPU-local dense attention"; Alg. 2,
 * gpu_attention): softmax attention of each query head over ALL valid tokens
 * of `window`, which the caller has already extended with the token being
 * decoded.  Writes o_out [B,Hq,d] and lse_out [B,Hq] (fp32); both NULL defers
 * the result (see hgca_lse_merge_splits). */
int hgca_dense_window_attn(const hgca_shape *shape, const void *q,
                           const hgca_kv_view *window,
                           float *o_out, float *lse_out,
                           void *ws, size_t ws_bytes, void *hip_stream);

/* hgca_dense_window_attn for callers that cannot allocate device memory or
 * bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels and same result as
 * hgca_dense_window_attn with o_out and lse_out given (both are required
 * here), but the split partials live in a device array that is part of the
 * library's code object (HGCA_STATIC_SCRATCH_BYTES on every GPU the library
 * runs on, held until the process ends) instead of in `ws`.  The call
 * allocates nothing and frees nothing; the first call on a device looks up
 * the address of that device's copy of the array.  Shapes whose partials do
 * not fit -- hgca_workspace_bytes(shape, window->cap, 0, 0) greater than
 * HGCA_STATIC_SCRATCH_BYTES -- are refused with HGCA_ERR_WORKSPACE and
 * nothing is enqueued.  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams) race; calls in stream order
 * do not, and nothing in the array needs clearing between calls. */
#define HGCA_STATIC_SCRATCH_BYTES (16u << 20)
int hgca_dense_window_attn_static(const hgca_shape *shape, const void *q,
                                  const hgca_kv_view *window,
                                  float *o_out, float *lse_out,
                                  void *hip_stream);

/* Raw attention scores of the older context (Sec. 3.3, s_j = q . k_j; what
 * Alg. 2's cpu_attention hands to the re-evaluation as A_cpu, before the
 * softmax): scores_out[b,h,t] = sm_scale * <q[b,h], K[b,h/G,t]> for every valid
 * token t of `pool`; scores_out is fp32 [B,Hq,pool->cap], entries at
 * t >= seq_lens[b] are left untouched.  Only pool->k is read.  This is the first
 * pass of hgca_select_salient, exposed on its own. */
int hgca_pool_scores(const hgca_shape *shape, const void *q,
                     const hgca_kv_view *pool, float *scores_out,
                     void *hip_stream);

/* Per-head selection of salient entries of the older context (Sec. 3.2.2,
 * head-granularity sparsification; fixed-budget top-k form of Sec. 2.2):
 * for every (b, h) score every valid pool token with the current query and keep
 * the k_b = min(k, len_b) highest scores, k = k_per_seq[b] (device [B]) if
 * given, else k_uniform.  Equal scores: the lower position wins.  Scores are
 * compared in fp32.  idx_out [B,Hq,k_max] receives the kept logical positions in
 * ascending order, padded with -1; cnt_out [B,Hq] receives k_b.  k_max is the
 * row length of idx_out: min(k_uniform, pool->cap) must not exceed it (checked
 * on the host; per-sequence budgets are clamped to k_max on the device).
 * sel_scores_out (optional, NULL to skip) is fp32 [B,Hq,k_max] and receives the
 * score s_j of every kept entry, in the order of idx_out (entries at or beyond
 * cnt are left untouched).  Only pool->k is read. */
int hgca_select_salient(const hgca_shape *shape, const void *q,
                        const hgca_kv_view *pool,
                        const int32_t *k_per_seq, int32_t k_uniform,
                        int32_t k_max, int32_t *idx_out, int32_t *cnt_out,
                        float *sel_scores_out,
                        void *ws, size_t ws_bytes, void *hip_stream);

/* The second pass of hgca_select_salient on scores the caller supplies (Sec.
 * 3.2.2: the sparsifier ranks entries by a per-head relevance value, which may
 * as well be the moving average of attention weights that hgca_maw_update
 * keeps): per (b, h) row of scores (device fp32 [B,Hq,cap], 16-byte aligned;
 * +inf and -inf are ordinary values here, e.g. -inf for positions a caller has
 * masked: they rank above / below every finite score, ties among them by
 * position; with NaN the selection is unspecified) keep
 * the k_b = min(k, len_b) largest of the first len_b = seq_lens[b] entries (all
 * `cap` if seq_lens is NULL).  Tie rule, budgets,
 * k_max, idx_out, cnt_out and sel_scores_out as in hgca_select_salient.  Only
 * batch and n_q_heads of `shape` are used. */
int hgca_select_topk(const hgca_shape *shape, const float *scores,
                     const int32_t *seq_lens, int32_t cap,
                     const int32_t *k_per_seq, int32_t k_uniform,
                     int32_t k_max, int32_t *idx_out, int32_t *cnt_out,
                     float *sel_scores_out, void *hip_stream);

/* Per-head sparse attention (Sec. 3.3 "CPU-local sparse attention"; Alg. 2,
 * cpu_attention): softmax attention of query head (b,h) over pool rows
 * idx[b,h,0 .. cnt[b,h]).  Entries at or beyond cnt[b,h] are ignored; the
 * listed positions must be valid and distinct (a repeated position is counted
 * twice; a position outside [0, pool->cap) is read as the nearest one inside,
 * so the result is meaningless but nothing outside the tier is touched).  Writes o_out [B,Hq,d] and lse_out [B,Hq] (fp32); both NULL defers
 * the result (see hgca_lse_merge_splits).
 * sel_scores (optional, NULL for none) is fp32 [B,Hq,k_max] holding the score
 * s_j = sm_scale * <q, k_j> of every listed entry for THIS q, as
 * hgca_select_salient returns it: the scores are then taken as given and the
 * K rows are not read again (only pool->v is).  Pass NULL whenever q differs
 * from the query the scores were computed for. */
int hgca_sparse_attn(const hgca_shape *shape, const void *q,
                     const hgca_kv_view *pool,
                     const int32_t *idx, const int32_t *cnt, int32_t k_max,
                     const float *sel_scores,
                     float *o_out, float *lse_out,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* Deferred results.  hgca_dense_window_attn and hgca_sparse_attn are split-K
 * kernels followed by a small fold of the splits.  Called with o_out == NULL and
 * lse_out == NULL (both), they skip the fold and leave their split partials in
 * `ws`; hgca_lse_merge_splits then folds the splits of BOTH parts in one kernel,
 * which is merge_state (Sec. 3.3 "Merging states") applied to all partial states at
 * once -- the fusion is associative -- and saves two kernel launches per step.
 * window_cap and k_max must be the window->cap and k_max of the two deferred calls
 * (they fix the split counts), ws_dense / ws_sparse the workspaces those calls
 * used, untouched since; either may be NULL for "no such part".  o_out is
 * [B,Hq,d] in o_dtype (fp32 or bf16), lse_out [B,Hq] fp32 or NULL. */
int hgca_lse_merge_splits(const hgca_shape *shape,
                          int32_t window_cap, const void *ws_dense, size_t ws_dense_bytes,
                          int32_t k_max, const void *ws_sparse, size_t ws_sparse_bytes,
                          void *o_out, int32_t o_dtype, float *lse_out,
                          void *hip_stream);

/* The whole decode branch of Alg. 2 in one call: dense window part, per-head
 * top-k selection over the pool with the current query (as
 * hgca_select_salient), sparse part over the selected entries, merge_state.
 * Same results as hgca_dense_window_attn + hgca_select_salient +
 * hgca_sparse_attn (with the selection's scores) + hgca_lse_merge_splits (the
 * same selection; O and lse up to the order of the fp32 sums), for one
 * crossing of the boundary: the kept entries' scores stay in the workspace
 * and one fold produces O.  idx_out / cnt_out receive
 * the selection (reusable by later steps through hgca_sparse_attn); o_out is
 * [B,Hq,d] in o_dtype, lse_out [B,Hq] optional.  ws_dense needs
 * hgca_workspace_bytes(shape, window->cap, 0, 0), ws_sparse
 * hgca_workspace_bytes(shape, 0, pool->cap, k_max); they must be different
 * buffers. */
int hgca_hybrid_decode_step(const hgca_shape *shape, const void *q,
                            const hgca_kv_view *window, const hgca_kv_view *pool,
                            const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max,
                            int32_t *idx_out, int32_t *cnt_out,
                            void *o_out, int32_t o_dtype, float *lse_out,
                            void *ws_dense, size_t ws_dense_bytes,
                            void *ws_sparse, size_t ws_sparse_bytes,
                            void *hip_stream);

/* The decode branch of Alg. 2 as the paper runs it for every token: the salient
 * entries are already selected (kv_manager.load returns KV_ctx), so the step is
 * gpu_attention over the window beside cpu_attention over each head's listed
 * entries, then merge_state.  Same results as hgca_dense_window_attn and
 * hgca_sparse_attn with deferred results + hgca_lse_merge_splits (up to the
 * order of the fp32 sums: the split sizes differ), in one crossing of the
 * boundary; the split kernels of the two parts, which need nothing from each
 * other, share one launch where the shapes allow.
 * idx / cnt / k_max / sel_scores as in hgca_sparse_attn (sel_scores NULL unless
 * it holds the scores of the listed entries for THIS q).  o_out is [B,Hq,d] in
 * o_dtype, lse_out [B,Hq] optional.  ws_dense needs
 * hgca_workspace_bytes(shape, window->cap, 0, 0), ws_sparse
 * hgca_workspace_bytes(shape, 0, 0, k_max); they must be different buffers. */
int hgca_hybrid_decode_step_selected(const hgca_shape *shape, const void *q,
                                     const hgca_kv_view *window, const hgca_kv_view *pool,
                                     const int32_t *idx, const int32_t *cnt, int32_t k_max,
                                     const float *sel_scores,
                                     void *o_out, int32_t o_dtype, float *lse_out,
                                     void *ws_dense, size_t ws_dense_bytes,
                                     void *ws_sparse, size_t ws_sparse_bytes,
                                     void *hip_stream);

/* merge_state (Sec. 3.3 "Merging states"): combines two partial results over
 * disjoint key sets into the result of one softmax over their union.  Evaluated
 * with both exponents shifted by max(lse_a, lse_b).  o_out is [B,Hq,d] in
 * o_dtype (fp32 or bf16) and may alias o_a or o_b when o_dtype is fp32 (the
 * paper merges in place); lse_out [B,Hq] is optional (NULL to skip) and may
 * alias lse_a or lse_b.  Only batch, n_q_heads and head_dim of `shape` are used. */
int hgca_lse_merge(const hgca_shape *shape,
                   const float *o_a, const float *lse_a,
                   const float *o_b, const float *lse_b,
                   void *o_out, int32_t o_dtype, float *lse_out,
                   void *hip_stream);

/* ---- The paper's own sparsifier: attention weights of the window, their
 * moving average, and the beta/size threshold rule (Alg. 1; Sec. 3.2.2). ---- */

/* hgca_dense_window_attn that also returns A_gpu (Alg. 2, gpu_attention returns
 * O_gpu, lse_g and A_gpu): a_out is fp32 [B,Hq,window->cap] and receives the
 * softmax weight e^{s_j - lse_g} of every valid window token (Sec. 2.1,
 * A = softmax(S)) and 0 at positions >= seq_lens[b].  o_out and lse_out are
 * required (the result cannot be deferred). */
int hgca_dense_window_attn_weights(const hgca_shape *shape, const void *q,
                                   const hgca_kv_view *window,
                                   float *o_out, float *lse_out, float *a_out,
                                   void *ws, size_t ws_bytes, void *hip_stream);

/* hgca_dense_window_attn_weights followed by hgca_maw_update(a_maw, a_out,
 * window->seq_lens, window->cap, n_new, alpha) in the same kernels (Alg. 2's
 * gpu_attention, then the first statement of Alg. 1): one launch and one pass
 * over the weights fewer per decode step.  a_maw is fp32 [B,Hq,window->cap],
 * updated in place; results are identical to the two separate calls. */
int hgca_dense_window_attn_maw(const hgca_shape *shape, const void *q,
                               const hgca_kv_view *window,
                               float *o_out, float *lse_out, float *a_out,
                               float *a_maw, int32_t n_new, float alpha,
                               void *ws, size_t ws_bytes, void *hip_stream);

/* Moving average of attention weights (Alg. 1, the A_maw update; Sec. 3.1):
 * a_maw <- (1 - alpha) * a_maw + alpha * a_gpu on the first seq_lens[b] entries
 * of every (b, h) row (all `cap` entries if seq_lens is NULL); a_maw and a_gpu
 * are device fp32 [B,Hq,cap], a_maw is updated in place, entries beyond the
 * length are left untouched.  The last n_new valid entries of a row (the tokens
 * appended since the previous update: 1 per decode step) have no history and
 * are set to a_gpu, their first observed weight.  0 <= alpha <= 1.  Only batch
 * and n_q_heads of `shape` are used. */
int hgca_maw_update(const hgca_shape *shape, float *a_maw, const float *a_gpu,
                    const int32_t *seq_lens, int32_t cap, int32_t n_new,
                    float alpha, void *hip_stream);

/* Per-head threshold rule (Sec. 3.2.2; Alg. 1, ids <- A > beta / A.size):
 * entry j of row (b, h) is salient iff weights[b,h,j] > beta / size_b
 * (strictly), size_b = size_per_seq[b] (device [B]) if given, else
 * size_uniform (> 0): the number of entries the weights were taken over.
 * The comparison is made in fp64 on the exactly widened fp32 weight.  weights
 * is device fp32 [B,Hq,cap]; the first seq_lens[b] entries of a row are
 * examined (all if seq_lens is NULL).  idx_out [B,Hq,k_max] receives the
 * salient positions in ascending order, padded with -1, cnt_out [B,Hq] their
 * number; if more than k_max entries pass, the first k_max in position order
 * are kept and cnt_out is k_max (pass k_max = cap to rule that out).
 * w_norm_out (optional, NULL to skip) is fp32 [B,Hq,k_max] and receives the
 * kept weights re-normalised to sum to 1 per row, 0 in the padding.  The result
 * feeds hgca_sparse_attn as idx / cnt.  Only batch and n_q_heads of `shape` are
 * used. */
int hgca_threshold_select(const hgca_shape *shape, const float *weights,
                          const int32_t *seq_lens, int32_t cap,
                          const int32_t *size_per_seq, int32_t size_uniform,
                          double beta, int32_t k_max,
                          int32_t *idx_out, int32_t *cnt_out, float *w_norm_out,
                          void *hip_stream);

/* ---- Group-shared salient lists for grouped-query attention (Sec. 3.3, "CPU-local
 * sparse attention": adjacent heads are merged into one sparse attention task and
 * the per-head sparsification is relaxed: a merged head may be padded with
 * entries that do not meet its own criterion).  The heads of a GQA group read the
 * same K/V rows, so the merge unit here is the group: ONE list of pool positions
 * per KV head, idx [B,Hkv,k_max] / cnt [B,Hkv], attended by every head of the
 * group; the sparse part then reads each listed row once per group instead of
 * once per head. ---- */

/* Group budget: per (b, KV head) the k_b entries with the largest group score,
 * the group score of an entry being the maximum over the group's heads of
 * s_j = sm_scale * <q_h, k_j>.  Budgets, tie rule, k_max and outputs as in
 * hgca_select_salient, with Hkv rows per sequence instead of Hq. */
int hgca_select_salient_grouped(const hgca_shape *shape, const void *q,
                                const hgca_kv_view *pool,
                                const int32_t *k_per_seq, int32_t k_uniform,
                                int32_t k_max, int32_t *idx_out, int32_t *cnt_out,
                                void *ws, size_t ws_bytes, void *hip_stream);

/* Union: per (b, KV head) the ascending union of the lists idx [B,Hq,k_max] /
 * cnt [B,Hq] of the group's heads (nothing a head selected is lost).  Positions
 * lie in [0, n_positions), n_positions <= HGCA_UNION_MAX_POSITIONS (more is
 * HGCA_ERR_UNSUPPORTED).  idx_out is [B,Hkv,k_max_out],
 * -1 padded, cnt_out [B,Hkv]; a union longer than k_max_out is cut (lowest
 * positions kept) and bit 0 of *status (device int32, optional) is set. */
#define HGCA_UNION_MAX_POSITIONS 523776
int hgca_union_lists(const hgca_shape *shape, const int32_t *idx, const int32_t *cnt,
                     int32_t k_max, int32_t n_positions,
                     int32_t *idx_out, int32_t *cnt_out, int32_t k_max_out,
                     int32_t *status, void *hip_stream);

/* hgca_sparse_attn with one list per KV head: query head (b,h) attends to pool
 * rows idx[b, h/G, 0 .. cnt[b, h/G]).  Outputs, deferral and workspace as in
 * hgca_sparse_attn (k_max fixes the split count the same way). */
int hgca_sparse_attn_grouped(const hgca_shape *shape, const void *q,
                             const hgca_kv_view *pool,
                             const int32_t *idx, const int32_t *cnt, int32_t k_max,
                             float *o_out, float *lse_out,
                             void *ws, size_t ws_bytes, void *hip_stream);

/* ---- KV manager across decode steps (Alg. 1; Sec. 3.2.1 retention and
 * offload, Sec. 3.2.2 sparsification). ----
 *
 * In the paper the recent window is a circular buffer of fixed-size blocks in
 * GPU memory and evicted blocks are copied to host memory.  Here both tiers are
 * ranges of ONE per-sequence list of blocks in HBM: row b of `block_table`
 * names, in arrival order, the physical blocks of sequence b; the older pool is
 * its first first_win_block[b] blocks, the window the blocks after them.
 * Evicting the oldest window block therefore moves a boundary and copies no KV
 * row.  Views for the attention calls:
 *   window = { k_blocks, v_blocks, win_lens,  block_table, cap = window capacity
 *              (see win_cap_blocks), block_size, max_blocks, first_block =
 *              first_win_block }
 *   pool   = { k_blocks, v_blocks, pool_lens, block_table, cap = pool_cap,
 *              block_size, max_blocks, first_block = NULL }
 * All pointers are device memory owned by the caller; the struct itself is host
 * memory read during the call.  Arrays marked (rw) are updated by the calls. */
typedef struct {
    void          *k_blocks, *v_blocks; /* [n_blocks, Hkv, block_size, d], dtype of the shape (rw) */
    const int32_t *block_table;         /* [B, max_blocks]: blocks of each sequence, oldest first   */
    int32_t       *first_win_block;     /* [B] (rw) first window block = number of pool blocks      */
    int32_t       *win_lens;            /* [B] (rw) tokens in the window                            */
    int32_t       *pool_lens;           /* [B] (rw) tokens in the pool = first_win_block*block_size */
    float         *a_maw;               /* [B, Hq, window capacity] (rw) moving average of          */
                                        /* attention weights, by window position                    */
    int32_t       *ctx_idx;             /* [B, Hq, k_max] (rw) salient pool positions, ascending    */
    int32_t       *ctx_cnt;             /* [B, Hq] (rw) their number                                */
    float         *a_evicted;           /* optional [B, Hq, pool_cap] (rw): moving average of every */
                                        /* evicted entry at its pool position; NULL to skip         */
    int32_t       *plan;                /* [B, 4] (rw) scratch of hgca_kv_evict: zero before the    */
                                        /* first call, left with [.,3] = 0 by every call            */
    int32_t       *status;              /* [1] (rw) sticky HGCA_CACHE_* bits, 0 = consistent        */
    int32_t block_size;                 /* tokens per block, a multiple of 16                       */
    int32_t max_blocks;                 /* row length of block_table                                */
    int32_t win_blocks;                 /* blk_num of Alg. 1: l_max = win_blocks * block_size       */
    int32_t k_max;                      /* row length of ctx_idx                                    */
    int32_t pool_cap;                   /* capacity of the pool view and row length of a_evicted    */
    int32_t win_cap_blocks;             /* blocks the window may hold for a moment, >= win_blocks   */
                                        /* (0 counts as win_blocks): window capacity = row length   */
                                        /* of a_maw = win_cap_blocks * block_size tokens.  A decode */
                                        /* step needs no more than l_max; a prompt of N tokens      */
                                        /* needs l_max - 1 + N, until its eviction has run          */
} hgca_cache_state;

enum {
    HGCA_CACHE_WINDOW_FULL = 1,   /* insertion beyond the window's capacity: the tokens were dropped      */
    HGCA_CACHE_CONTEXT_FULL = 2,  /* append beyond the last block of the table row: token dropped        */
    HGCA_CACHE_LIST_FULL = 4      /* more salient entries than k_max: the later ones were not listed     */
};

/* Insert the new token's KV entry (Alg. 1, KV_gpu.add(KV_in); Alg. 2 does it
 * before gpu_attention so that the window includes the token being decoded):
 * k_in, v_in are [B, Hkv, d] in shape.dtype, 16-byte aligned; the rows go to
 * window position win_lens[b], then win_lens[b] grows by one.  `active`
 * (device [B] or NULL = all) masks sequences that receive no token.  A full
 * window or table row sets a status bit and drops the token (call hgca_kv_evict
 * after every step and it cannot happen before the context is exhausted). */
int hgca_kv_append(const hgca_shape *shape, const hgca_cache_state *cache,
                   const void *k_in, const void *v_in, const int32_t *active,
                   void *hip_stream);

/* hgca_kv_append for a prompt: n_tokens entries per sequence at once (Alg. 1
 * with KV_in.size = N).  k_in, v_in are [B, n_tokens, Hkv, d], oldest first; they
 * go to window positions win_lens[b] .. win_lens[b] + n_tokens - 1.  A sequence
 * whose window capacity or table row cannot take all of them receives none
 * (status bit). */
int hgca_kv_append_tokens(const hgca_shape *shape, const hgca_cache_state *cache,
                          const void *k_in, const void *v_in, int32_t n_tokens,
                          const int32_t *active, void *hip_stream);

/* Eviction and sparsification of Alg. 1, per sequence, decided on the device:
 * if l_cur = win_lens[b] >= l_max, the oldest l_evict = ceil((l_cur - l_max + 1)
 * / block_size) * block_size window entries (the printed formula has l_max and
 * l_cur swapped) become the newest pool entries; for every head the evicted
 * entries with a_maw > beta / l_cur (strictly; fp64 comparison; A_gpu.size =
 * l_cur) are appended to ctx_idx as pool positions and the rest of the a_maw row
 * shifts down by l_evict (vacated entries become 0).  Call it after
 * hgca_maw_update of the step.  Sequences below l_max are left untouched. */
int hgca_kv_evict(const hgca_shape *shape, const hgca_cache_state *cache,
                  double beta, void *hip_stream);

/* One decode step over the managed cache in one call, in the paper's order:
 * Alg. 2, decode branch (KV_gpu' = concat(KV_gpu, KV_in); gpu_attention over
 * the window, which returns A_gpu; cpu_attention over each head's salient
 * entries KV_ctx; merge_state), then Alg. 1 (A_maw <- (1 - alpha) A_maw + alpha
 * A_gpu, the inserted token taking its first observed weight; eviction and
 * sparsification with beta where a window has reached l_max).  The same
 * results as hgca_kv_append, hgca_dense_window_attn_maw, hgca_sparse_attn on
 * (ctx_idx, ctx_cnt), hgca_lse_merge_splits and hgca_kv_evict in that order,
 * in two launches where the shapes allow (bf16, groups of 1, 2 or 4): the
 * window split that owns the token's position writes its rows, the splits of
 * window and salient lists share the launch, and one launch per (sequence,
 * head) row folds the partials, forms A_gpu with the window's own lse from
 * the same fold, updates A_maw, evicts and stores the window's new length.
 * If the token does not fit (status bits as for hgca_kv_append) the step runs
 * on the window as it stands.  q is [B,Hq,d], k_in / v_in [B,Hkv,d]: every sequence of the
 * batch receives a token (batches in which some do not use the separate
 * calls); a_gpu (device fp32 [B,Hq,window capacity], required)
 * receives A_gpu; o_out [B,Hq,d] in o_dtype, lse_out
 * [B,Hq] optional.  ws_dense needs hgca_workspace_bytes(shape, window capacity,
 * 0, 0), ws_sparse hgca_workspace_bytes(shape, 0, 0, k_max);
 * different buffers.  Every decision is taken on the device: the launch
 * sequence is the same every step. */
int hgca_managed_decode_step(const hgca_shape *shape, const hgca_cache_state *cache,
                             const void *q, const void *k_in, const void *v_in,
                             float alpha, double beta,
                             float *a_gpu, void *o_out, int32_t o_dtype, float *lse_out,
                             void *ws_dense, size_t ws_dense_bytes,
                             void *ws_sparse, size_t ws_sparse_bytes, void *hip_stream);

/* One append turn over the managed cache in one call (a prompt of n_q tokens per
 * sequence), in the paper's order: Alg. 2, append branch -- KV_gpu' =
 * concat(KV_gpu, KV_in); gpu_attention over the window, causal among the
 * incoming tokens; cpu_attention over the COMPLETE offloaded cache (not the
 * salient lists); merge_state per query -- then Alg. 1 with KV_in.size = n_q:
 * the moving averages are updated with the query-averaged A_gpu (the n_q new
 * entries take their first observed weight); the salient lists are REPLACED by
 * the re-evaluation of Sec. 3.2.2, ids = A_cpu > beta / A_cpu.size with A_cpu the
 * query-averaged weights over the offloaded cache and A_cpu.size = pool_lens[b];
 * then windows that have reached l_max evict as many whole blocks as it takes,
 * their salient entries joining the new lists.  The same results as
 * hgca_kv_append_tokens, hgca_append_attn on the window (causal tail) and on the
 * pool, hgca_lse_merge, hgca_append_weights on both, hgca_maw_update (n_new =
 * n_q), hgca_threshold_select on a_cpu and hgca_kv_evict in that order.
 * q is [B, n_q, Hq, d], k_in / v_in [B, n_q, Hkv, d] (dtypes as hgca_append_attn);
 * flags: HGCA_APPEND_ONE_PART_P or 0; a_gpu (fp32 [B,Hq,window capacity]) and
 * a_cpu (fp32 [B,Hq,pool_cap]) receive the two weight rows (0 beyond the
 * lengths); o_out is fp32 [B,n_q,Hq,d], lse_out fp32
 * [B,n_q,Hq].  The window capacity must take l_cur = win_lens[b] + n_q (see
 * win_cap_blocks).  `ws` needs hgca_managed_append_workspace_bytes. */
size_t hgca_managed_append_workspace_bytes(const hgca_shape *shape, const hgca_cache_state *cache,
                                           int32_t n_q);
int hgca_managed_append_step(const hgca_shape *shape, const hgca_cache_state *cache,
                             const void *q, const void *k_in, const void *v_in, int32_t n_q,
                             float alpha, double beta, int32_t flags,
                             float *a_gpu, float *a_cpu, float *o_out, float *lse_out,
                             void *ws, size_t ws_bytes, void *hip_stream);

/* KV_ctx of Alg. 1 (KV_ctx.add(KV_evict[ids]); Sec. 3.2.2): per head, the
 * salient entries held in contiguous storage, so that the sparse part reads a
 * stream instead of following an index list.  For every (b, h) the K and V
 * rows of pool positions idx[b,h,0..cnt[b,h]) (valid positions, as for
 * hgca_sparse_attn) are copied, bit for bit and in list order, to rows
 * first_row[b,h] + j of k_ctx / v_ctx [B, Hq, ctx_cap, d] (shape.dtype,
 * 16-byte aligned, two different buffers).  first_row (device [B,Hq]) may be
 * NULL = 0; rows that would land at ctx_cap or beyond are left out.  cnt_out
 * (device [B,Hq], optional, not the same array as first_row or cnt) receives
 * min(first_row + cnt, ctx_cap): pass it as first_row of the next call to add
 * the entries of a later eviction behind the earlier ones.
 * Attention over KV_ctx is hgca_dense_window_attn on the shape {batch = B*Hq,
 * n_q_heads = 1, n_kv_heads = 1} with the view {k_ctx, v_ctx, seq_lens =
 * cnt_out, cap = ctx_cap}: every head is a sequence of its own. */
int hgca_ctx_compact(const hgca_shape *shape, const hgca_kv_view *pool,
                     const int32_t *idx, const int32_t *cnt, int32_t k_max,
                     const int32_t *first_row, void *k_ctx, void *v_ctx,
                     int32_t ctx_cap, int32_t *cnt_out, void *hip_stream);

/* ---- Append stage (Sec. 2.1: N incoming tokens, Q in R^{h x N x d}; Alg. 2,
 * append branch).  bf16 inputs run both contractions on the matrix cores;
 * fp32 inputs (the exact shapes) run on the vector units: every (sequence,
 * query) pair is then a one-query attention over the tokens that query sees,
 * served by the split kernels of the decode path (B * n_q <= 65 535). ----
 *
 * q is [B, N, Hq, d].  Attention of all N queries over one tier; the two parts
 * of the hybrid step are two calls (the window with HGCA_APPEND_CAUSAL_TAIL,
 * the complete older pool without) whose results hgca_lse_merge combines with
 * a shape whose batch is B*N.  `flags` is a sum of:
 * HGCA_APPEND_CAUSAL_TAIL: the tier's last N valid tokens are the incoming
 * tokens themselves and attention among them is causal: query i (0-based) sees
 * tokens [0, seq_lens[b] - N + i + 1).  Without it every query sees every valid
 * token.
 * HGCA_APPEND_ONE_PART_P: the softmax weights enter the second contraction
 * rounded once to bf16 (relative error 2^-9 per weight: |dO| <= 2^-9 max|v|,
 * typically ~1e-3 for unit-variance V; lse unaffected), a third fewer matrix
 * instructions.  Without it they enter as a high and a low bf16 part and O
 * keeps fp32-level accuracy (~1e-6).  (Ignored for fp32 inputs, whose weights
 * stay fp32 throughout.)
 * Other bits are rejected.  shape.sm_scale must be positive and finite for the
 * append entry points.  o_out is fp32 [B, N, Hq, d], lse_out fp32
 * [B, N, Hq]; a query that sees nothing gives O = 0, lse = -inf.  ws needs
 * hgca_append_workspace_bytes(shape, n_q, tier->cap) bytes.  n_q <= 4096. */
enum {
    HGCA_APPEND_CAUSAL_TAIL = 1,
    HGCA_APPEND_ONE_PART_P = 2
};
size_t hgca_append_workspace_bytes(const hgca_shape *shape, int32_t n_q,
                                   int32_t max_tokens);
int hgca_append_attn(const hgca_shape *shape, const void *q, int32_t n_q,
                     const hgca_kv_view *tier, int32_t flags,
                     float *o_out, float *lse_out,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* Both parts of the append branch of Alg. 2 in one call: attention of the N
 * queries over the window (HGCA_APPEND_CAUSAL_TAIL in `flags` applies to the
 * window) and over the COMPLETE older pool, merged per (sequence, query, head)
 * with merge_state.  The same results as hgca_append_attn on each tier and
 * hgca_lse_merge (up to the order of fp32 additions), in two launches instead
 * of five: the splits of both tiers share one launch and one split size, and
 * one fold of all split partials yields the merged output together with each
 * tier's own log-sum-exp.  o_out fp32 [B, N, Hq, d], lse_out fp32 [B, N, Hq];
 * lse_window_out / lse_pool_out (fp32 [B, N, Hq], optional) receive the
 * per-tier lse that hgca_append_weights normalises with.  bf16 inputs only
 * (HGCA_ERR_UNSUPPORTED for fp32: use the per-tier calls).  ws needs
 * hgca_append_tiers_workspace_bytes(shape, n_q, window->cap, pool->cap). */
size_t hgca_append_tiers_workspace_bytes(const hgca_shape *shape, int32_t n_q,
                                         int32_t window_cap, int32_t pool_cap);
int hgca_append_attn_tiers(const hgca_shape *shape, const void *q, int32_t n_q,
                           const hgca_kv_view *window, const hgca_kv_view *pool,
                           int32_t flags, float *o_out, float *lse_out,
                           float *lse_window_out, float *lse_pool_out,
                           void *ws, size_t ws_bytes, void *hip_stream);

/* A_gpu / A_cpu of the append branch (Alg. 2 returns them; Alg. 1 re-evaluates
 * the salient set with ids = A_cpu > beta / A_cpu.size): one weight per head
 * and entry, the average over the N queries of the part's own softmax weights,
 * a_out[b,h,t] = (1/N) * sum_i e^{s_it - lse[b,i,h]} over the queries i that
 * see t, where lse is the lse_out of hgca_append_attn on the same tier (same q,
 * n_q, causal_tail != 0 iff HGCA_APPEND_CAUSAL_TAIL there).  a_out is fp32
 * [B, Hq, tier->cap], 0 at t >= seq_lens[b].  Only tier->k is read. */
int hgca_append_weights(const hgca_shape *shape, const void *q, int32_t n_q,
                        const hgca_kv_view *tier, int32_t causal_tail,
                        const float *lse, float *a_out, void *hip_stream);

/* The same for both tiers of an append turn in one launch (bf16 inputs;
 * HGCA_ERR_UNSUPPORTED for fp32: one call per tier): a_gpu [B,Hq,window->cap]
 * from lse_window (causal_tail applies to the window), a_cpu [B,Hq,pool->cap]
 * from lse_pool, as hgca_append_attn_tiers returns them.  A tier of capacity 0
 * is skipped (its pointers may be NULL). */
int hgca_append_weights_tiers(const hgca_shape *shape, const void *q, int32_t n_q,
                              const hgca_kv_view *window, const hgca_kv_view *pool,
                              int32_t causal_tail, const float *lse_window,
                              const float *lse_pool, float *a_gpu, float *a_cpu,
                              void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HGCA_H */
