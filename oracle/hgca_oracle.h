/*
 * CPU oracle for HGCA decode-time hybrid attention (arXiv 2507.03153).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 reference written
 * from the paper's equations.  It shares no code with the HIP library and is
 * never called by it; only the test-suite, the smoke check and the benchmark's
 * CPU-baseline leg may use it.
 *
 * What it computes (paper notation):
 *   - softmax attention of one decode query per head over a key set I
 *     (Sec. 2.1: S = QK^T, A = softmax(S), O = AV), together with
 *     lse_I = log sum_{j in I} exp(s_j)            (Sec. 3.3, "Merging states");
 *   - the GPU-local dense part: I = the W most recent tokens (Sec. 3.3,
 *     "GPU-local dense attention"; Alg. 2, gpu_attention);
 *   - the per-head sparse part: I = each head's own selected subset of the
 *     offloaded context (Sec. 3.3, "CPU-local sparse attention"; Alg. 2,
 *     cpu_attention);
 *   - per-head selection of salient offloaded entries (Sec. 3.2.2,
 *     head-granularity sparsification), in the fixed-budget top-k form the
 *     paper describes in Sec. 2.2: the k entries with the largest attention
 *     score of the current query;
 *   - merge_state: z = e^{lse_c} + e^{lse_g},
 *     O = (e^{lse_c} O_cpu + e^{lse_g} O_gpu) / z   (Sec. 3.3, merge equations);
 *   - the paper's own sparsifier: the window's attention weights A_gpu, their
 *     moving average (Alg. 1: A_maw <- (1-alpha) A_maw + alpha A_gpu) and the
 *     per-head threshold rule "keep iff weight > beta / size" (Sec. 3.2.2).
 *
 * Readings taken where the paper is silent:
 *   - scores are scaled, s_j = scale * <q, k_j>, scale is an argument;
 *   - log is the natural logarithm;
 *   - query head h reads KV head h / (Hq / Hkv)  (contiguous groups);
 *   - the merge is evaluated with both exponents shifted by max(lse), which is
 *     the same value as the printed formula and cannot overflow;
 *   - an empty set has O = 0 and lse = -inf;
 *   - selection ranks by score, higher first, equal scores by lower position;
 *     the selected positions are reported in ascending order;
 *     k_b = min(k, P_b).
 *
 * Every function is pinned by tests that run without a GPU (closed forms,
 * library softmax / logsumexp / argsort, pure-Python brute force, the union
 * identity of the merge, and "select everything == full attention").
 *
 * Layouts.  q is [B, Hq, d].  A KV tier is either contiguous,
 * k/v = [B, Hkv, cap, d] with the valid tokens of sequence b at positions
 * [0, len_b), or paged, k/v = [n_blocks, Hkv, block_size, d] with logical
 * token t of sequence b stored in physical block block_table[b, t / block_size]
 * at slot t % block_size.  Elements are fp32, or bf16 given as raw 16-bit
 * patterns (widened exactly).  All arithmetic is fp64.
 */
#ifndef HGCA_ORACLE_H
#define HGCA_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

typedef struct {
    int32_t dtype;          /* ORACLE_F32 or ORACLE_BF16 (for q, K and V) */
    int32_t batch;          /* B   */
    int32_t n_q_heads;      /* Hq  */
    int32_t n_kv_heads;     /* Hkv, divides Hq */
    int32_t head_dim;       /* d   */
    double  scale;          /* multiplies <q,k> before the softmax */
} oracle_shape;

typedef struct {
    const void    *k, *v;
    const int32_t *seq_lens;     /* [B] valid tokens; NULL => cap for all */
    const int32_t *block_table;  /* [B, max_blocks]; NULL => contiguous   */
    int32_t cap, block_size, max_blocks;
} oracle_kv;

/* Scaled scores s_j of every valid token of the tier, per query head.
 * scores is [B, Hq, cap]; positions >= len_b are set to -inf. */
int oracle_scores(const oracle_shape *sh, const void *q, const oracle_kv *kv,
                  double *scores);

/* Attention over all valid tokens [0, len_b) of one tier (the dense window).
 * o is [B, Hq, d], lse is [B, Hq]. */
int oracle_attend_all(const oracle_shape *sh, const void *q,
                      const oracle_kv *kv, double *o, double *lse);

/* Attention over rows idx[b, h, 0 .. cnt[b,h]) of one tier (the per-head
 * sparse part).  idx is [B, Hq, k_max] (logical token positions). */
int oracle_attend_indexed(const oracle_shape *sh, const void *q,
                          const oracle_kv *kv, const int32_t *idx,
                          const int32_t *cnt, int32_t k_max,
                          double *o, double *lse);

/* One-pass attention over (all valid tokens of `window`) U (rows idx of
 * `pool`); idx == NULL means every valid pool token.  This is the "single
 * softmax over the union" the merge is required to equal. */
int oracle_attend_union(const oracle_shape *sh, const void *q,
                        const oracle_kv *window, const oracle_kv *pool,
                        const int32_t *idx, const int32_t *cnt, int32_t k_max,
                        double *o, double *lse);

/* Per-head top-k of the pool by score.  k for sequence b is
 * min(k_per_seq ? k_per_seq[b] : k_uniform, len_b).  round_scores_to_f32 != 0
 * rounds each fp64 score to fp32 before ranking (the precision in which the
 * HIP path takes the same decision).  idx is [B, Hq, k_max], filled ascending,
 * padded with -1; cnt is [B, Hq]. */
int oracle_select(const oracle_shape *sh, const void *q, const oracle_kv *pool,
                  const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max,
                  int round_scores_to_f32, int32_t *idx, int32_t *cnt);

/* The same ranking (score descending, lower position first on ties, output
 * ascending) on caller-supplied scores [rows, cap]; lens and k per ROW. */
int oracle_select_given(int64_t rows, int32_t cap, const int32_t *lens,
                        const int32_t *k_per_row, int32_t k_uniform, int32_t k_max,
                        const double *scores, int32_t *idx, int32_t *cnt);

/* merge_state on n_rows independent (batch, head) rows of width d. */
int oracle_merge(int64_t n_rows, int32_t d,
                 const double *o_a, const double *lse_a,
                 const double *o_b, const double *lse_b,
                 double *o, double *lse);

/* The whole layer-step in the order of Alg. 2's decode branch: dense window,
 * selection, sparse part, merge.  select != 0 runs the selection (writing
 * idx/cnt); select == 0 reuses the idx/cnt passed in. */
int oracle_hybrid_step(const oracle_shape *sh, const void *q,
                       const oracle_kv *window, const oracle_kv *pool,
                       const int32_t *k_per_seq, int32_t k_uniform,
                       int32_t k_max, int select, int32_t *idx, int32_t *cnt,
                       double *o, double *lse);

/* ---- the paper's own sparsifier (Alg. 1; Sec. 3.2.2) ---- */

/* A_gpu of Alg. 2: softmax weights of the query over the dense window,
 * a is [B, Hq, cap], zero at positions >= len_b. */
int oracle_window_weights(const oracle_shape *sh, const void *q,
                          const oracle_kv *kv, double *a);

/* Alg. 1: A_maw <- (1-alpha) A_maw + alpha A_gpu, rows = B*Hq of [cap] entries,
 * lens per ROW (NULL => cap); the last n_new valid entries of a row take their
 * first observed weight. */
int oracle_maw_update(int64_t rows, int32_t cap, const int32_t *lens,
                      int32_t n_new, double alpha, double *maw, const double *a);

/* Sec. 3.2.2: keep iff w > beta / size (strict); sizes per ROW or uniform.
 * idx [rows, k_max] ascending, -1 padded (first k_max passing entries if more
 * pass), cnt [rows]; w_norm optional [rows, k_max]: kept weights re-normalised
 * to sum to 1 per row. */
int oracle_threshold_select(int64_t rows, int32_t cap, const int32_t *lens,
                            const int32_t *sizes, int32_t size_uniform,
                            double beta, const double *w, int32_t k_max,
                            int32_t *idx, int32_t *cnt, double *w_norm);

/* Number of OpenMP threads the (batch, head) loop will use. */
int oracle_num_threads(void);
/* Threads the (batch, head) loops may use from now on (timing of the baseline on 1 core and on all cores). */
void oracle_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
