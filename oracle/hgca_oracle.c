/*
 * CPU oracle for HGCA decode-time hybrid attention -- see hgca_oracle.h.
 * TEST INFRASTRUCTURE ONLY; fp64 throughout; no blocking, fusion or
 * reordering beyond what the definitions state.  The only parallelism is one
 * task per (batch, head), the decomposition Sec. 3.3 ("CPU-local sparse
 * attention") gives.
 */
#include "hgca_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- element access ---------------------------------------------------- */

static double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    /* bf16 is the upper half of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int32_t seq_len(const oracle_kv *kv, int b)
{
    return kv->seq_lens ? kv->seq_lens[b] : kv->cap;
}

/* element offset of row (b, kvh, t) inside kv->k / kv->v */
static size_t row_offset(const oracle_shape *sh, const oracle_kv *kv,
                         int b, int kvh, int32_t t)
{
    size_t d = (size_t)sh->head_dim, H = (size_t)sh->n_kv_heads;
    if (kv->block_table) {
        size_t blk = (size_t)kv->block_table[(size_t)b * kv->max_blocks
                                             + t / kv->block_size];
        size_t slot = (size_t)(t % kv->block_size);
        return ((blk * H + kvh) * kv->block_size + slot) * d;
    }
    return (((size_t)b * H + kvh) * kv->cap + t) * d;
}

static int shape_ok(const oracle_shape *sh)
{
    return sh && sh->batch >= 0 && sh->n_q_heads > 0 && sh->n_kv_heads > 0
        && sh->head_dim > 0 && sh->n_q_heads % sh->n_kv_heads == 0
        && (sh->dtype == ORACLE_F32 || sh->dtype == ORACLE_BF16);
}

/* s = scale * <q[b,h,:], K[b,kvh(h),t,:]>   (Sec. 3.3: s_j = q . k_j) */
static double score_of(const oracle_shape *sh, const void *q,
                       const oracle_kv *kv, int b, int h, int32_t t)
{
    int d = sh->head_dim;
    int kvh = h / (sh->n_q_heads / sh->n_kv_heads);
    size_t qo = ((size_t)b * sh->n_q_heads + h) * d;
    size_t ko = row_offset(sh, kv, b, kvh, t);
    double acc = 0.0;
    for (int c = 0; c < d; ++c)
        acc += load_elem(q, sh->dtype, qo + c) * load_elem(kv->k, sh->dtype, ko + c);
    return sh->scale * acc;
}

/* ---- softmax attention over an explicit list of (tier, token) ---------- */

typedef struct { const oracle_kv *kv; int32_t t; } key_ref;

/* Sec. 2.1 restricted to the set: A = softmax(s), O = A V; lse = log sum e^s.
 * Evaluated as m = max s, l = sum e^{s-m}, lse = m + log l. */
static void attend_set(const oracle_shape *sh, const void *q, int b, int h,
                       const key_ref *set, size_t n, double *o, double *lse)
{
    int d = sh->head_dim;
    int kvh = h / (sh->n_q_heads / sh->n_kv_heads);
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (n == 0) { *lse = -INFINITY; return; }

    double *s = (double *)malloc(n * sizeof *s);
    double m = -INFINITY;
    for (size_t j = 0; j < n; ++j) {
        s[j] = score_of(sh, q, set[j].kv, b, h, set[j].t);
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (size_t j = 0; j < n; ++j) l += exp(s[j] - m);
    for (size_t j = 0; j < n; ++j) {
        double a = exp(s[j] - m) / l;                 /* softmax weight */
        size_t vo = row_offset(sh, set[j].kv, b, kvh, set[j].t);
        for (int c = 0; c < d; ++c)
            o[c] += a * load_elem(set[j].kv->v, sh->dtype, vo + c);
    }
    *lse = m + log(l);
    free(s);
}

/* ---- public entry points ------------------------------------------------ */

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_scores(const oracle_shape *sh, const void *q, const oracle_kv *kv,
                  double *scores)
{
    if (!shape_ok(sh) || !q || !kv || !scores) return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t n = seq_len(kv, b);
        double *row = scores + (size_t)bh * kv->cap;
        for (int32_t t = 0; t < kv->cap; ++t)
            row[t] = t < n ? score_of(sh, q, kv, b, h, t) : -INFINITY;
    }
    return 0;
}

int oracle_attend_all(const oracle_shape *sh, const void *q,
                      const oracle_kv *kv, double *o, double *lse)
{
    if (!shape_ok(sh) || !q || !kv || !o || !lse) return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t n = seq_len(kv, b);
        key_ref *set = (key_ref *)malloc(((size_t)n + 1) * sizeof *set);
        for (int32_t t = 0; t < n; ++t) { set[t].kv = kv; set[t].t = t; }
        attend_set(sh, q, b, h, set, (size_t)n,
                   o + (size_t)bh * sh->head_dim, lse + bh);
        free(set);
    }
    return 0;
}

int oracle_attend_indexed(const oracle_shape *sh, const void *q,
                          const oracle_kv *kv, const int32_t *idx,
                          const int32_t *cnt, int32_t k_max,
                          double *o, double *lse)
{
    if (!shape_ok(sh) || !q || !kv || !idx || !cnt || !o || !lse || k_max < 0)
        return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t n = cnt[bh];
        if (n < 0 || n > k_max) { bad = 1; continue; }
        key_ref *set = (key_ref *)malloc(((size_t)n + 1) * sizeof *set);
        for (int32_t j = 0; j < n; ++j) {
            int32_t t = idx[(size_t)bh * k_max + j];
            if (t < 0 || t >= seq_len(kv, b)) bad = 1;
            set[j].kv = kv; set[j].t = t;
        }
        if (!bad)
            attend_set(sh, q, b, h, set, (size_t)n,
                       o + (size_t)bh * sh->head_dim, lse + bh);
        free(set);
    }
    return bad ? -2 : 0;
}

int oracle_attend_union(const oracle_shape *sh, const void *q,
                        const oracle_kv *window, const oracle_kv *pool,
                        const int32_t *idx, const int32_t *cnt, int32_t k_max,
                        double *o, double *lse)
{
    if (!shape_ok(sh) || !q || !window || !pool || !o || !lse) return -1;
    if (idx && !cnt) return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t nw = seq_len(window, b);
        int32_t np = idx ? cnt[bh] : seq_len(pool, b);
        key_ref *set = (key_ref *)malloc(((size_t)nw + np + 1) * sizeof *set);
        for (int32_t t = 0; t < nw; ++t) { set[t].kv = window; set[t].t = t; }
        for (int32_t j = 0; j < np; ++j) {
            set[nw + j].kv = pool;
            set[nw + j].t = idx ? idx[(size_t)bh * k_max + j] : j;
        }
        attend_set(sh, q, b, h, set, (size_t)nw + np,
                   o + (size_t)bh * sh->head_dim, lse + bh);
        free(set);
    }
    return 0;
}

/* ranking order of the selection: higher score first, then lower position */
typedef struct { double s; int32_t t; } scored;

static int by_score_desc_then_pos(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->t > b->t) - (a->t < b->t);
}

static int by_int32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

int oracle_select(const oracle_shape *sh, const void *q, const oracle_kv *pool,
                  const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max,
                  int round_scores_to_f32, int32_t *idx, int32_t *cnt)
{
    if (!shape_ok(sh) || !q || !pool || !idx || !cnt || k_max < 0) return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t n = seq_len(pool, b);
        int32_t k = k_per_seq ? k_per_seq[b] : k_uniform;
        if (k < 0) { bad = 1; k = 0; }
        if (k > n) k = n;
        if (k > k_max) { bad = 1; k = k_max; }
        int32_t *out = idx + (size_t)bh * k_max;

        scored *all = (scored *)malloc(((size_t)n + 1) * sizeof *all);
        for (int32_t t = 0; t < n; ++t) {
            double s = score_of(sh, q, pool, b, h, t);
            if (round_scores_to_f32) s = (double)(float)s;
            all[t].s = s; all[t].t = t;
        }
        qsort(all, (size_t)n, sizeof *all, by_score_desc_then_pos);
        for (int32_t j = 0; j < k; ++j) out[j] = all[j].t;
        qsort(out, (size_t)k, sizeof *out, by_int32);
        for (int32_t j = k; j < k_max; ++j) out[j] = -1;
        cnt[bh] = k;
        free(all);
    }
    return bad ? -2 : 0;
}

/* The same ranking on scores the caller supplies (for instance moving averages
 * of attention weights): rows of [cap] doubles, lens / k per ROW. */
int oracle_select_given(int64_t rows, int32_t cap, const int32_t *lens,
                        const int32_t *k_per_row, int32_t k_uniform, int32_t k_max,
                        const double *scores, int32_t *idx, int32_t *cnt)
{
    if (rows < 0 || cap < 0 || k_max < 0 || !scores || !idx || !cnt) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        int32_t n = lens ? lens[r] : cap;
        int32_t k = k_per_row ? k_per_row[r] : k_uniform;
        if (k > n) k = n;
        if (k > k_max) k = k_max;
        if (k < 0) k = 0;
        int32_t *out = idx + (size_t)r * k_max;
        scored *all = (scored *)malloc(((size_t)n + 1) * sizeof *all);
        for (int32_t t = 0; t < n; ++t) { all[t].s = scores[(size_t)r * cap + t]; all[t].t = t; }
        qsort(all, (size_t)n, sizeof *all, by_score_desc_then_pos);
        for (int32_t j = 0; j < k; ++j) out[j] = all[j].t;
        qsort(out, (size_t)k, sizeof *out, by_int32);
        for (int32_t j = k; j < k_max; ++j) out[j] = -1;
        cnt[r] = k;
        free(all);
    }
    return 0;
}

int oracle_merge(int64_t n_rows, int32_t d,
                 const double *o_a, const double *lse_a,
                 const double *o_b, const double *lse_b,
                 double *o, double *lse)
{
    if (n_rows < 0 || d <= 0 || !o_a || !lse_a || !o_b || !lse_b || !o)
        return -1;
    for (int64_t r = 0; r < n_rows; ++r) {
        double la = lse_a[r], lb = lse_b[r];
        double m = la > lb ? la : lb;
        if (m == -INFINITY) {                       /* both sets empty */
            for (int c = 0; c < d; ++c) o[r * d + c] = 0.0;
            if (lse) lse[r] = -INFINITY;
            continue;
        }
        /* e^{lse}/z with both exponents shifted by m */
        double ea = exp(la - m), eb = exp(lb - m), z = ea + eb;
        for (int c = 0; c < d; ++c)
            o[r * d + c] = (ea * o_a[r * d + c] + eb * o_b[r * d + c]) / z;
        if (lse) lse[r] = m + log(z);
    }
    return 0;
}

int oracle_hybrid_step(const oracle_shape *sh, const void *q,
                       const oracle_kv *window, const oracle_kv *pool,
                       const int32_t *k_per_seq, int32_t k_uniform,
                       int32_t k_max, int select, int32_t *idx, int32_t *cnt,
                       double *o, double *lse)
{
    if (!shape_ok(sh) || !o || !lse || !idx || !cnt) return -1;
    size_t n_bh = (size_t)sh->batch * sh->n_q_heads, d = (size_t)sh->head_dim;
    double *o_g = (double *)malloc((n_bh * d + 1) * sizeof(double));
    double *o_c = (double *)malloc((n_bh * d + 1) * sizeof(double));
    double *l_g = (double *)malloc((n_bh + 1) * sizeof(double));
    double *l_c = (double *)malloc((n_bh + 1) * sizeof(double));
    int rc = oracle_attend_all(sh, q, window, o_g, l_g);
    if (!rc && select)
        rc = oracle_select(sh, q, pool, k_per_seq, k_uniform, k_max, 1, idx, cnt);
    if (!rc) rc = oracle_attend_indexed(sh, q, pool, idx, cnt, k_max, o_c, l_c);
    if (!rc) rc = oracle_merge((int64_t)n_bh, sh->head_dim, o_c, l_c, o_g, l_g, o, lse);
    free(o_g); free(o_c); free(l_g); free(l_c);
    return rc;
}

/* ---- the paper's own sparsifier (Alg. 1; Sec. 3.2.2) ---------------------- */

/* A = softmax(S) of Sec. 2.1 for the dense window: the A_gpu that Alg. 2's
 * gpu_attention returns.  a is [B, Hq, cap]; positions >= len_b are set to 0. */
int oracle_window_weights(const oracle_shape *sh, const void *q,
                          const oracle_kv *kv, double *a)
{
    if (!shape_ok(sh) || !q || !kv || !a) return -1;
    long n_bh = (long)sh->batch * sh->n_q_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < n_bh; ++bh) {
        int b = (int)(bh / sh->n_q_heads), h = (int)(bh % sh->n_q_heads);
        int32_t n = seq_len(kv, b);
        double *row = a + (size_t)bh * kv->cap;
        double m = -INFINITY, l = 0.0;
        for (int32_t t = 0; t < n; ++t) {
            row[t] = score_of(sh, q, kv, b, h, t);
            if (row[t] > m) m = row[t];
        }
        for (int32_t t = 0; t < n; ++t) l += exp(row[t] - m);
        for (int32_t t = 0; t < n; ++t) row[t] = exp(row[t] - m) / l;
        for (int32_t t = n; t < kv->cap; ++t) row[t] = 0.0;
    }
    return 0;
}

/* Alg. 1: A_maw <- (1 - alpha) * A_maw + alpha * A_gpu for every GPU-resident
 * entry of every head.  maw and a are [rows, cap]; lens[r] entries of row r are
 * valid; the last n_new valid entries of a row have no history yet and take
 * their first observed weight (a reading: the paper does not say). */
int oracle_maw_update(int64_t rows, int32_t cap, const int32_t *lens,
                      int32_t n_new, double alpha, double *maw, const double *a)
{
    if (rows < 0 || cap < 0 || n_new < 0 || !maw || !a) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        int32_t n = lens ? lens[r] : cap;
        for (int32_t t = 0; t < n; ++t) {
            size_t i = (size_t)r * cap + t;
            maw[i] = (t >= n - n_new) ? a[i] : (1.0 - alpha) * maw[i] + alpha * a[i];
        }
    }
    return 0;
}

/* Sec. 3.2.2: an entry is salient for a head iff its weight exceeds beta / size
 * (strictly), size being the number of entries the weights were taken over.
 * w is [rows, cap]; kept positions go to idx [rows, k_max] in ascending order
 * (-1 padded; if more than k_max pass, the first k_max in position order are
 * kept), their count to cnt [rows].  w_norm (optional, [rows, k_max]) receives
 * the kept weights re-normalised to sum to 1 per row, as the paper does after
 * selection. */
int oracle_threshold_select(int64_t rows, int32_t cap, const int32_t *lens,
                            const int32_t *sizes, int32_t size_uniform,
                            double beta, const double *w, int32_t k_max,
                            int32_t *idx, int32_t *cnt, double *w_norm)
{
    if (rows < 0 || cap < 0 || k_max < 0 || !w || !idx || !cnt) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        int32_t n = lens ? lens[r] : cap;
        int32_t size = sizes ? sizes[r] : size_uniform;
        double thr = beta / (double)size;
        int32_t kept = 0;
        double sum = 0.0;
        for (int32_t t = 0; t < n && kept < k_max; ++t) {
            double x = w[(size_t)r * cap + t];
            if (x > thr) {
                idx[(size_t)r * k_max + kept] = t;
                if (w_norm) w_norm[(size_t)r * k_max + kept] = x;
                sum += x;
                ++kept;
            }
        }
        for (int32_t j = kept; j < k_max; ++j) {
            idx[(size_t)r * k_max + j] = -1;
            if (w_norm) w_norm[(size_t)r * k_max + j] = 0.0;
        }
        if (w_norm)
            for (int32_t j = 0; j < kept; ++j) w_norm[(size_t)r * k_max + j] /= sum;
        cnt[r] = kept;
    }
    return 0;
}
