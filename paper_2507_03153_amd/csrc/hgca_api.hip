// C ABI of libhgca: argument validation, workspace layout, kernel sequencing.
// See include/hgca.h for the contract of every entry point.
#include "../../include/hgca.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>

#include "hgca_launch.hpp"

namespace {

using namespace hgca;

constexpr size_t kAlign = 256;
// Workgroups a launch aims for (256 CUs): compile-time tunables, one per streaming pass.
#ifndef HGCA_TARGET_WGS_DENSE_SHARED
#define HGCA_TARGET_WGS_DENSE_SHARED 512
#endif
#ifndef HGCA_TARGET_WGS_DENSE
#define HGCA_TARGET_WGS_DENSE 1024
#endif
#ifndef HGCA_TARGET_WGS_SCORES
#define HGCA_TARGET_WGS_SCORES 32768
#endif
#ifndef HGCA_TARGET_WGS_SPARSE
#define HGCA_TARGET_WGS_SPARSE 2048
#endif
#ifndef HGCA_TARGET_WGS_SPARSE_SCORED            // the sparse part inside hgca_hybrid_decode_step (scores given, V only)
#define HGCA_TARGET_WGS_SPARSE_SCORED 2048
#endif

// workgroups the append-stage weights pass aims at (its tokens per workgroup are halved from 2048 until it has them)
#ifndef HGCA_WEIGHTS_TARGET_WGS
#define HGCA_WEIGHTS_TARGET_WGS 1024
#endif
// Workgroups the append-stage attention aims at per launch: what the device holds at once (two per compute unit).
// Every workgroup writes a partial of 128 rows x d floats (64 KB, read again by the fold: the K/V bytes of four
// 64-token steps), so splits are as long as filling the device allows.  Measured on the 8B shape, N = 32, with
// 512 / 768 / 1024 / 1536: window 55.7 / 61.0 / 66.0 / 74.8 us, pool 258.5 / 273.4 / 266.6 / 288.1 us.
#ifndef HGCA_APPEND_TARGET_WGS
#define HGCA_APPEND_TARGET_WGS 512
#endif
// 1: moving average, re-evaluation and eviction of an append turn are one launch
#ifndef HGCA_FUSE_APPEND_TAIL
#define HGCA_FUSE_APPEND_TAIL 1
#endif
// 1: the token of a managed decode step is written into the window by the window split that reads it (needs the two below)
#ifndef HGCA_FUSE_KV_APPEND
#define HGCA_FUSE_KV_APPEND 1
#endif
// 1: the tail of the managed decode step (fold, window weights + moving average, eviction) is one launch
#ifndef HGCA_FUSE_DECODE_TAIL
#define HGCA_FUSE_DECODE_TAIL 1
#endif
// 1: the window's split kernels and the sparse part's split kernels of a step share a launch where the shapes allow
#ifndef HGCA_FUSE_DENSE_GATHER
#define HGCA_FUSE_DENSE_GATHER 1
#endif

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int group_of(const hgca_shape *s) { return s->n_q_heads / s->n_kv_heads; }

int check_shape(const hgca_shape *s)
{
    if (!s) return HGCA_ERR_INVALID_ARG;
    if (s->batch < 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0) return HGCA_ERR_INVALID_ARG;
    if (s->n_q_heads % s->n_kv_heads != 0) return HGCA_ERR_INVALID_ARG;
    // sequences and heads are grid dimensions y and z of the launches (65 535 at most each)
    if (s->batch > 65535 || s->n_q_heads > 65535) return HGCA_ERR_UNSUPPORTED;
    if (s->dtype != HGCA_F32 && s->dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (s->head_dim != 64 && s->head_dim != 128) return HGCA_ERR_UNSUPPORTED;
    const int g = group_of(s);
    if (g != 1 && g != 2 && g != 4 && g != 8) return HGCA_ERR_UNSUPPORTED;
    if (!(s->sm_scale == s->sm_scale)) return HGCA_ERR_INVALID_ARG;   // NaN
    return HGCA_OK;
}

int check_view(const hgca_shape *s, const hgca_kv_view *v, bool need_v)
{
    if (!v) return HGCA_ERR_INVALID_ARG;
    if (v->cap < 0) return HGCA_ERR_INVALID_ARG;
    // rows of a tier are numbered with 32 bits inside the kernels
    if (!v->block_table && (int64_t)s->batch * s->n_kv_heads * v->cap >= (int64_t(1) << 32)) return HGCA_ERR_UNSUPPORTED;
    if (v->cap > 0) {
        if (!v->k || !aligned16(v->k)) return HGCA_ERR_INVALID_ARG;
        if (need_v && (!v->v || !aligned16(v->v))) return HGCA_ERR_INVALID_ARG;
    }
    if (v->block_table) {
        if (v->block_size <= 0 || v->max_blocks <= 0) return HGCA_ERR_INVALID_ARG;
        if (v->block_size % 16 != 0) return HGCA_ERR_UNSUPPORTED;
        if ((int64_t)v->max_blocks * v->block_size < v->cap) return HGCA_ERR_INVALID_ARG;
    }
    return HGCA_OK;
}

KvDev to_dev(const hgca_kv_view *v)
{
    KvDev d{};
    d.k = static_cast<const char *>(v->k);
    d.v = static_cast<const char *>(v->v);
    d.seq_lens = v->seq_lens;
    d.block_table = v->block_table;
    d.first_block = v->block_table ? v->first_block : nullptr;
    d.cap = v->cap;
    d.block_size = v->block_table ? v->block_size : 1;
    d.max_blocks = v->block_table ? v->max_blocks : 0;
    return d;
}

ShapeDev to_dev(const hgca_shape *s)
{
    ShapeDev d{};
    d.batch = s->batch;
    d.n_q_heads = s->n_q_heads;
    d.n_kv_heads = s->n_kv_heads;
    d.group = group_of(s);
    d.sm_scale = s->sm_scale;
    return d;
}

// Tokens per split for a set of at most n tokens processed by `units` independent
// (sequence, head unit) pairs: a multiple of 64 in [kMinChunk, kMaxChunk] that yields
// roughly `target` workgroups.
int pick_chunk(int64_t n, int64_t units, int target, int max_chunk = kMaxChunk)
{
    if (n <= 0 || units <= 0) return kMinChunk;
    const int64_t want_splits = std::max<int64_t>(1, target / units);
    int64_t chunk = (n + want_splits - 1) / want_splits;
    chunk = (chunk + 63) / 64 * 64;
    return (int)std::min<int64_t>(max_chunk, std::max<int64_t>(kMinChunk, chunk));
}

int n_splits_for(int64_t n, int chunk) { return (int)((n + chunk - 1) / chunk); }

// Tokens per window split: in a launch of its own the window wants about HGCA_TARGET_WGS_DENSE workgroups; in a launch
// it shares with the sparse part's splits, which fill the device anyway, longer splits (half as many partials to write
// and fold) are better.  Measured on the 8B shape: full step 145.2 -> 143.8 us, steady 67.9 -> 67.6 us; on its own the
// window is 1 us slower with them.
int dense_chunk(const hgca_shape *s, int64_t cap, bool shares_launch)
{
    return pick_chunk(cap, (int64_t)s->batch * s->n_kv_heads, shares_launch ? HGCA_TARGET_WGS_DENSE_SHARED : HGCA_TARGET_WGS_DENSE);
}

// Tokens per workgroup of the score pass over a pool of `cap` tokens.  Groups of 8 heads take half the tokens per
// workgroup (64 instead of 128 on the 70B shape: 317 against 321 us per step).
int score_chunk(const hgca_shape *s, int64_t cap)
{
    const int target = HGCA_TARGET_WGS_SCORES * (s->n_q_heads / s->n_kv_heads >= 8 ? 2 : 1);
    return pick_chunk(cap, (int64_t)s->batch * s->n_kv_heads, target, s->dtype == HGCA_BF16 ? kMaxScoreChunk : kMaxChunk);
}

// Workspace layout: [partials o | partials m | partials l | one float per row | scores | scores of the kept entries].
struct WsLayout {
    size_t part_o, part_m, part_l, row_aux, scores, sel, total;
};

WsLayout layout(const hgca_shape *s, int64_t max_attn_tokens, int64_t max_pool)
{
    const size_t rows = (size_t)s->batch * s->n_q_heads;
    const size_t max_splits = (size_t)n_splits_for(std::max<int64_t>(max_attn_tokens, 1), kMinChunk);
    WsLayout w{};
    size_t at = 0;
    w.part_o = at; at += align_up(rows * max_splits * s->head_dim * sizeof(float));
    w.part_m = at; at += align_up(rows * max_splits * sizeof(float));
    w.part_l = at; at += align_up(rows * max_splits * sizeof(float));
    w.row_aux = at; at += align_up(rows * sizeof(float));
    w.scores = at; at += align_up(rows * (size_t)std::max<int64_t>(max_pool, 0) * sizeof(float));
    w.sel = at; at += max_pool > 0 ? align_up(rows * (size_t)std::max<int64_t>(max_attn_tokens, 0) * sizeof(float)) : 0;
    w.total = std::max<size_t>(at, kAlign);
    return w;
}

Partials partials_at(void *ws, const WsLayout &w, int n_splits)
{
    char *base = static_cast<char *>(ws);
    Partials p{};
    p.o = reinterpret_cast<float *>(base + w.part_o);
    p.m = reinterpret_cast<float *>(base + w.part_m);
    p.l = reinterpret_cast<float *>(base + w.part_l);
    p.n_splits = n_splits;
    return p;
}

int from_hip(hipError_t e) { return e == hipSuccess ? HGCA_OK : HGCA_ERR_DEVICE; }

}  // namespace

extern "C" {

const char *hgca_status_string(int status)
{
    switch (status) {
    case HGCA_OK: return "ok";
    case HGCA_ERR_INVALID_ARG: return "invalid argument";
    case HGCA_ERR_UNSUPPORTED: return "unsupported shape, dtype or layout";
    case HGCA_ERR_WORKSPACE: return "workspace missing or too small";
    case HGCA_ERR_DEVICE: return "HIP launch failed";
    default: return "unknown status";
    }
}

size_t hgca_workspace_bytes(const hgca_shape *shape, int32_t max_window, int32_t max_pool, int32_t k_max)
{
    if (check_shape(shape) != HGCA_OK || max_window < 0 || max_pool < 0 || k_max < 0) return 0;
    return layout(shape, std::max(max_window, k_max), max_pool).total;
}

namespace {

int dense_window(const hgca_shape *shape, const void *q, const hgca_kv_view *window, float *o_out, float *lse_out,
                 float *a_out, float *a_maw, int32_t n_new, float alpha, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;       // nothing to do
    if ((rc = check_view(shape, window, true)) != HGCA_OK) return rc;
    const bool deferred = !o_out && !lse_out;    // leave the split partials in ws for hgca_lse_merge_splits
    if (!q || !aligned16(q) || (!deferred && (!o_out || !lse_out || !aligned16(o_out)))) return HGCA_ERR_INVALID_ARG;
    if (a_out && deferred) return HGCA_ERR_INVALID_ARG;   // the weights need the window's own lse
    const WsLayout w = layout(shape, window->cap, 0);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    AttnArgs a{};
    a.sh = to_dev(shape);
    a.q = q;
    a.kv = to_dev(window);
    a.chunk = pick_chunk(window->cap, (int64_t)shape->batch * shape->n_kv_heads, HGCA_TARGET_WGS_DENSE);
    a.part = partials_at(ws, w, n_splits_for(window->cap, a.chunk));
    a.raw_scores = a_out;
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    if ((rc = from_hip(launch_attn_partial_dense(shape->dtype, shape->head_dim, a, s))) != HGCA_OK) return rc;
    if (deferred) return HGCA_OK;
    if ((rc = from_hip(launch_combine(shape->head_dim, rows, a.part, o_out, lse_out, s))) != HGCA_OK) return rc;
    if (!a_out) return HGCA_OK;
    return from_hip(launch_window_weights(a_out, lse_out, window->seq_lens, rows, shape->n_q_heads, window->cap, a_maw,
                                          n_new, alpha, s));
}

}  // namespace

int hgca_dense_window_attn(const hgca_shape *shape, const void *q, const hgca_kv_view *window, float *o_out,
                           float *lse_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return dense_window(shape, q, window, o_out, lse_out, nullptr, nullptr, 0, 0.f, ws, ws_bytes, hip_stream);
}

}  // extern "C"

// ---- dense window attention for callers that cannot allocate ---------------------------------------------
// The split partials of the call live in a file-scope device array instead of a caller's workspace.  Its name is
// a host-side stand-in here, not a device address: the address of each device's copy comes from
// hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[HGCA_STATIC_SCRATCH_BYTES];

namespace {

// Device address of the current device's copy of `scratch`; NULL (and *err set) if the runtime refuses.
void *static_scratch(hipError_t *err)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> known[kMaxDevices];               // zero-initialised
    int dev = 0;
    if ((*err = hipGetDevice(&dev)) != hipSuccess) return nullptr;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    void *ptr = tracked ? known[dev].load(std::memory_order_acquire) : nullptr;
    if (!ptr) {
        if ((*err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess) return nullptr;
        if (tracked) known[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

}  // namespace

extern "C" {

int hgca_dense_window_attn_static(const hgca_shape *shape, const void *q, const hgca_kv_view *window, float *o_out,
                                  float *lse_out, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, window, true)) != HGCA_OK) return rc;
    if (!o_out || !lse_out) return HGCA_ERR_INVALID_ARG;         // no deferred result: the partials are not the caller's
    if (layout(shape, window->cap, 0).total > (size_t)HGCA_STATIC_SCRATCH_BYTES) return HGCA_ERR_WORKSPACE;
    hipError_t err = hipSuccess;
    void *ws = static_scratch(&err);
    if (!ws) return HGCA_ERR_DEVICE;
    // every split writes its whole partial (empty ones included) and the fold reads only those, so nothing in the
    // array has to be cleared between calls
    return dense_window(shape, q, window, o_out, lse_out, nullptr, nullptr, 0, 0.f, ws, HGCA_STATIC_SCRATCH_BYTES,
                        hip_stream);
}

int hgca_dense_window_attn_weights(const hgca_shape *shape, const void *q, const hgca_kv_view *window, float *o_out,
                                   float *lse_out, float *a_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!a_out && window && window->cap > 0) return HGCA_ERR_INVALID_ARG;
    return dense_window(shape, q, window, o_out, lse_out, a_out, nullptr, 0, 0.f, ws, ws_bytes, hip_stream);
}

int hgca_dense_window_attn_maw(const hgca_shape *shape, const void *q, const hgca_kv_view *window, float *o_out,
                               float *lse_out, float *a_out, float *a_maw, int32_t n_new, float alpha, void *ws,
                               size_t ws_bytes, void *hip_stream)
{
    if (window && window->cap > 0 && (!a_out || !a_maw)) return HGCA_ERR_INVALID_ARG;
    if (n_new < 0 || !(alpha >= 0.f && alpha <= 1.f)) return HGCA_ERR_INVALID_ARG;
    return dense_window(shape, q, window, o_out, lse_out, a_out, a_maw, n_new, alpha, ws, ws_bytes, hip_stream);
}

int hgca_maw_update(const hgca_shape *shape, float *a_maw, const float *a_gpu, const int32_t *seq_lens, int32_t cap,
                    int32_t n_new, float alpha, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (cap < 0 || n_new < 0 || !(alpha >= 0.f && alpha <= 1.f)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0 || cap == 0) return HGCA_OK;
    if (!a_maw || !a_gpu) return HGCA_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_maw_update(a_maw, a_gpu, seq_lens, rows, shape->n_q_heads, cap, n_new, alpha,
                                      static_cast<hipStream_t>(hip_stream)));
}

int hgca_threshold_select(const hgca_shape *shape, const float *weights, const int32_t *seq_lens, int32_t cap,
                          const int32_t *size_per_seq, int32_t size_uniform, double beta, int32_t k_max,
                          int32_t *idx_out, int32_t *cnt_out, float *w_norm_out, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (cap < 0 || k_max < 0 || !(beta >= 0.0) || (!size_per_seq && size_uniform <= 0)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0) return HGCA_OK;
    if (!cnt_out || (k_max > 0 && !idx_out) || (cap > 0 && !weights)) return HGCA_ERR_INVALID_ARG;
    ThresholdArgs a{};
    a.w = weights;
    a.seq_lens = seq_lens;
    a.sizes = size_per_seq;
    a.beta = beta;
    a.size_uniform = size_uniform;
    a.n_q_heads = shape->n_q_heads;
    a.cap = cap;
    a.k_max = k_max;
    a.idx = idx_out;
    a.cnt = cnt_out;
    a.w_norm = k_max > 0 ? w_norm_out : nullptr;
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_threshold_select(a, rows, static_cast<hipStream_t>(hip_stream)));
}

int hgca_pool_scores(const hgca_shape *shape, const void *q, const hgca_kv_view *pool, float *scores_out,
                     void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, false)) != HGCA_OK) return rc;
    if (!q || !aligned16(q) || (pool->cap > 0 && (!scores_out || !aligned16(scores_out)))) return HGCA_ERR_INVALID_ARG;
    ScoreArgs sa{};
    sa.sh = to_dev(shape);
    sa.q = q;
    sa.kv = to_dev(pool);
    sa.scores = scores_out;
    sa.chunk = score_chunk(shape, pool->cap);
    sa.n_chunks = n_splits_for(pool->cap, sa.chunk);
    return from_hip(launch_scores(shape->dtype, shape->head_dim, sa, static_cast<hipStream_t>(hip_stream)));
}

int hgca_select_salient(const hgca_shape *shape, const void *q, const hgca_kv_view *pool, const int32_t *k_per_seq,
                        int32_t k_uniform, int32_t k_max, int32_t *idx_out, int32_t *cnt_out,
                        float *sel_scores_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, false)) != HGCA_OK) return rc;
    if (!q || !aligned16(q) || !cnt_out || k_max < 0 || (k_max > 0 && !idx_out)) return HGCA_ERR_INVALID_ARG;
    if (!k_per_seq && (k_uniform < 0 || std::min(k_uniform, pool->cap) > k_max)) return HGCA_ERR_INVALID_ARG;
    const WsLayout w = layout(shape, 0, pool->cap);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    ScoreArgs sa{};
    sa.sh = to_dev(shape);
    sa.q = q;
    sa.kv = to_dev(pool);
    sa.scores = reinterpret_cast<float *>(static_cast<char *>(ws) + w.scores);
    sa.chunk = score_chunk(shape, pool->cap);
    sa.n_chunks = n_splits_for(pool->cap, sa.chunk);
    if ((rc = from_hip(launch_scores(shape->dtype, shape->head_dim, sa, s))) != HGCA_OK) return rc;

    SelectArgs se{};
    se.sh = sa.sh;
    se.kv = sa.kv;
    se.scores = sa.scores;
    se.k_per_seq = k_per_seq;
    se.k_uniform = k_uniform;
    se.k_max = k_max;
    se.idx = idx_out;
    se.cnt = cnt_out;
    se.sel_scores = sel_scores_out;
    return from_hip(launch_select(se, s));
}

int hgca_select_topk(const hgca_shape *shape, const float *scores, const int32_t *seq_lens, int32_t cap,
                     const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max, int32_t *idx_out, int32_t *cnt_out,
                     float *sel_scores_out, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (cap < 0 || k_max < 0) return HGCA_ERR_INVALID_ARG;
    if (!k_per_seq && (k_uniform < 0 || std::min(k_uniform, cap) > k_max)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0) return HGCA_OK;
    if (!cnt_out || (k_max > 0 && !idx_out) || (cap > 0 && (!scores || !aligned16(scores)))) return HGCA_ERR_INVALID_ARG;
    SelectArgs se{};
    se.sh = to_dev(shape);
    se.kv.seq_lens = seq_lens;
    se.kv.cap = cap;
    se.scores = scores;
    se.k_per_seq = k_per_seq;
    se.k_uniform = k_uniform;
    se.k_max = k_max;
    se.idx = idx_out;
    se.cnt = cnt_out;
    se.sel_scores = sel_scores_out;
    return from_hip(launch_select(se, static_cast<hipStream_t>(hip_stream)));
}

int hgca_sparse_attn(const hgca_shape *shape, const void *q, const hgca_kv_view *pool, const int32_t *idx,
                     const int32_t *cnt, int32_t k_max, const float *sel_scores, float *o_out, float *lse_out,
                     void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, true)) != HGCA_OK) return rc;
    const bool deferred = !o_out && !lse_out;
    if (!q || !aligned16(q) || (!deferred && (!o_out || !lse_out || !aligned16(o_out)))) return HGCA_ERR_INVALID_ARG;
    if (k_max < 0 || !cnt || (k_max > 0 && !idx)) return HGCA_ERR_INVALID_ARG;
    const WsLayout w = layout(shape, k_max, 0);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    AttnArgs a{};
    a.sh = to_dev(shape);
    a.q = q;
    a.kv = to_dev(pool);
    a.idx = idx;
    a.cnt = cnt;
    a.sel_scores = sel_scores;
    a.k_max = k_max;
    a.chunk = pick_chunk(k_max, (int64_t)shape->batch * shape->n_q_heads, HGCA_TARGET_WGS_SPARSE);
    a.part = partials_at(ws, w, std::max(1, n_splits_for(k_max, a.chunk)));
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    if ((rc = from_hip(launch_attn_partial_gather(shape->dtype, shape->head_dim, a, s))) != HGCA_OK) return rc;
    if (deferred) return HGCA_OK;
    return from_hip(launch_combine(shape->head_dim, rows, a.part, o_out, lse_out, s));
}

int hgca_select_salient_grouped(const hgca_shape *shape, const void *q, const hgca_kv_view *pool,
                                const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max, int32_t *idx_out,
                                int32_t *cnt_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, false)) != HGCA_OK) return rc;
    if (!q || !aligned16(q) || !cnt_out || k_max < 0 || (k_max > 0 && !idx_out)) return HGCA_ERR_INVALID_ARG;
    if (!k_per_seq && (k_uniform < 0 || std::min(k_uniform, pool->cap) > k_max)) return HGCA_ERR_INVALID_ARG;
    const WsLayout w = layout(shape, 0, pool->cap);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    ScoreArgs sa{};
    sa.sh = to_dev(shape);
    sa.q = q;
    sa.kv = to_dev(pool);
    sa.scores = reinterpret_cast<float *>(static_cast<char *>(ws) + w.scores);    // [B, Hkv, cap] of the region
    sa.group_max = 1;
    sa.chunk = score_chunk(shape, pool->cap);
    sa.n_chunks = n_splits_for(pool->cap, sa.chunk);
    if ((rc = from_hip(launch_scores(shape->dtype, shape->head_dim, sa, s))) != HGCA_OK) return rc;

    SelectArgs se{};
    se.sh = sa.sh;
    se.sh.n_q_heads = shape->n_kv_heads;         // one row of scores and one list per KV head
    se.kv = sa.kv;
    se.scores = sa.scores;
    se.k_per_seq = k_per_seq;
    se.k_uniform = k_uniform;
    se.k_max = k_max;
    se.idx = idx_out;
    se.cnt = cnt_out;
    return from_hip(launch_select(se, s));
}

int hgca_union_lists(const hgca_shape *shape, const int32_t *idx, const int32_t *cnt, int32_t k_max,
                     int32_t n_positions, int32_t *idx_out, int32_t *cnt_out, int32_t k_max_out, int32_t *status,
                     void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (k_max < 0 || k_max_out < 0 || n_positions < 0) return HGCA_ERR_INVALID_ARG;
    // one bit per position in the 64 KiB of LDS a kernel may use without asking for more (64 bytes of it are static)
    if (n_positions > HGCA_UNION_MAX_POSITIONS) return HGCA_ERR_UNSUPPORTED;
    if (shape->batch == 0) return HGCA_OK;
    if (!cnt || !cnt_out || (k_max > 0 && !idx) || (k_max_out > 0 && !idx_out)) return HGCA_ERR_INVALID_ARG;
    return from_hip(launch_union_lists(idx, cnt, k_max, shape->batch, shape->n_q_heads, shape->n_kv_heads, n_positions,
                                       idx_out, cnt_out, k_max_out, status, static_cast<hipStream_t>(hip_stream)));
}

int hgca_sparse_attn_grouped(const hgca_shape *shape, const void *q, const hgca_kv_view *pool, const int32_t *idx,
                             const int32_t *cnt, int32_t k_max, float *o_out, float *lse_out, void *ws,
                             size_t ws_bytes, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, true)) != HGCA_OK) return rc;
    const bool deferred = !o_out && !lse_out;
    if (!q || !aligned16(q) || (!deferred && (!o_out || !lse_out || !aligned16(o_out)))) return HGCA_ERR_INVALID_ARG;
    if (k_max < 0 || !cnt || (k_max > 0 && !idx)) return HGCA_ERR_INVALID_ARG;
    const WsLayout w = layout(shape, k_max, 0);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    AttnArgs a{};
    a.sh = to_dev(shape);
    a.q = q;
    a.kv = to_dev(pool);
    a.idx = idx;
    a.cnt = cnt;
    a.k_max = k_max;
    a.grouped = 1;
    // same split size as hgca_sparse_attn (hgca_lse_merge_splits derives the split count from k_max alone)
    a.chunk = pick_chunk(k_max, (int64_t)shape->batch * shape->n_q_heads, HGCA_TARGET_WGS_SPARSE);
    a.part = partials_at(ws, w, std::max(1, n_splits_for(k_max, a.chunk)));
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    if ((rc = from_hip(launch_attn_partial_gather(shape->dtype, shape->head_dim, a, s))) != HGCA_OK) return rc;
    if (deferred) return HGCA_OK;
    return from_hip(launch_combine(shape->head_dim, rows, a.part, o_out, lse_out, s));
}

int hgca_lse_merge_splits(const hgca_shape *shape, int32_t window_cap, const void *ws_dense, size_t ws_dense_bytes,
                          int32_t k_max, const void *ws_sparse, size_t ws_sparse_bytes, void *o_out, int32_t o_dtype,
                          float *lse_out, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (o_dtype != HGCA_F32 && o_dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (shape->batch == 0) return HGCA_OK;
    if (window_cap < 0 || k_max < 0 || !o_out || !aligned16(o_out)) return HGCA_ERR_INVALID_ARG;
    // the same layouts and split counts the two deferred calls used
    Partials pd{}, ps{};
    if (ws_dense) {
        const WsLayout w = layout(shape, window_cap, 0);
        if (ws_dense_bytes < w.total || !aligned16(ws_dense)) return HGCA_ERR_WORKSPACE;
        const int chunk = pick_chunk(window_cap, (int64_t)shape->batch * shape->n_kv_heads, HGCA_TARGET_WGS_DENSE);
        pd = partials_at(const_cast<void *>(ws_dense), w, n_splits_for(window_cap, chunk));
    }
    if (ws_sparse) {
        const WsLayout w = layout(shape, k_max, 0);
        if (ws_sparse_bytes < w.total || !aligned16(ws_sparse)) return HGCA_ERR_WORKSPACE;
        const int chunk = pick_chunk(k_max, (int64_t)shape->batch * shape->n_q_heads, HGCA_TARGET_WGS_SPARSE);
        ps = partials_at(const_cast<void *>(ws_sparse), w, std::max(1, n_splits_for(k_max, chunk)));
    }
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_combine2(shape->head_dim, rows, pd, ps, o_out, o_dtype, lse_out,
                                    static_cast<hipStream_t>(hip_stream)));
}

int hgca_hybrid_decode_step(const hgca_shape *shape, const void *q, const hgca_kv_view *window,
                            const hgca_kv_view *pool, const int32_t *k_per_seq, int32_t k_uniform, int32_t k_max,
                            int32_t *idx_out, int32_t *cnt_out, void *o_out, int32_t o_dtype, float *lse_out,
                            void *ws_dense, size_t ws_dense_bytes, void *ws_sparse, size_t ws_sparse_bytes,
                            void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (o_dtype != HGCA_F32 && o_dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, window, true)) != HGCA_OK) return rc;
    if ((rc = check_view(shape, pool, true)) != HGCA_OK) return rc;
    if (!q || !aligned16(q) || !o_out || !aligned16(o_out) || !cnt_out || k_max < 0 || (k_max > 0 && !idx_out))
        return HGCA_ERR_INVALID_ARG;
    if (!k_per_seq && (k_uniform < 0 || std::min(k_uniform, pool->cap) > k_max)) return HGCA_ERR_INVALID_ARG;
    const WsLayout wd = layout(shape, window->cap, 0);
    const WsLayout wsp = layout(shape, k_max, pool->cap);
    if (!ws_dense || ws_dense_bytes < wd.total || !aligned16(ws_dense)) return HGCA_ERR_WORKSPACE;
    if (!ws_sparse || ws_sparse_bytes < wsp.total || !aligned16(ws_sparse)) return HGCA_ERR_WORKSPACE;
    if (ws_dense == ws_sparse) return HGCA_ERR_WORKSPACE;       // the two parts are live at the same time
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    ScoreArgs sa{};
    sa.sh = to_dev(shape);
    sa.q = q;
    sa.kv = to_dev(pool);
    sa.scores = reinterpret_cast<float *>(static_cast<char *>(ws_sparse) + wsp.scores);
    sa.chunk = score_chunk(shape, pool->cap);
    sa.n_chunks = n_splits_for(pool->cap, sa.chunk);

    AttnArgs da{};
    da.sh = sa.sh;
    da.q = q;
    da.kv = to_dev(window);
    // The window's splits and the sparse part's splits are two streaming passes that need nothing from each other:
    // where the shapes allow they share one launch (after the selection), so the second needs no ramp-up of its own.
    const bool fuse_gather = HGCA_FUSE_DENSE_GATHER && pool->cap > 0 && window->cap > 0 && k_max > 0 &&
                             dense_gather_fusable(shape->dtype, shape->head_dim, group_of(shape));
    da.chunk = dense_chunk(shape, window->cap, fuse_gather);
    da.part = partials_at(ws_dense, wd, n_splits_for(window->cap, da.chunk));

    // 1. split kernels of the window part (unless they go with the sparse part's), score pass over the pool
    if (!fuse_gather && (rc = from_hip(launch_attn_partial_dense(shape->dtype, shape->head_dim, da, s))) != HGCA_OK)
        return rc;
    if ((rc = from_hip(launch_scores(shape->dtype, shape->head_dim, sa, s))) != HGCA_OK) return rc;
    // 2. per-head top-k; the kept entries' scores stay in the workspace for the sparse part
    float *sel = k_max > 0 && pool->cap > 0 ? reinterpret_cast<float *>(static_cast<char *>(ws_sparse) + wsp.sel) : nullptr;
    SelectArgs se{};
    se.sh = sa.sh;
    se.kv = sa.kv;
    se.scores = sa.scores;
    se.k_per_seq = k_per_seq;
    se.k_uniform = k_uniform;
    se.k_max = k_max;
    se.idx = idx_out;
    se.cnt = cnt_out;
    se.sel_scores = sel;
    if ((rc = from_hip(launch_select(se, s))) != HGCA_OK) return rc;
    // 3. sparse part on the given scores (V rows only)
    AttnArgs ga{};
    ga.sh = sa.sh;
    ga.q = q;
    ga.kv = sa.kv;
    ga.idx = idx_out;
    ga.cnt = cnt_out;
    ga.sel_scores = sel;
    ga.k_max = k_max;
    ga.chunk = pick_chunk(k_max, (int64_t)shape->batch * shape->n_q_heads, HGCA_TARGET_WGS_SPARSE_SCORED);
    ga.part = partials_at(ws_sparse, wsp, std::max(1, n_splits_for(k_max, ga.chunk)));
    if (fuse_gather) rc = from_hip(launch_dense_gather(shape->dtype, shape->head_dim, da, ga, s));
    else rc = from_hip(launch_attn_partial_gather(shape->dtype, shape->head_dim, ga, s));
    if (rc != HGCA_OK) return rc;
    // 4. one fold of all split partials = merge_state over all of them
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_combine2(shape->head_dim, rows, da.part, ga.part, o_out, o_dtype, lse_out, s));
}

int hgca_hybrid_decode_step_selected(const hgca_shape *shape, const void *q, const hgca_kv_view *window,
                                     const hgca_kv_view *pool, const int32_t *idx, const int32_t *cnt, int32_t k_max,
                                     const float *sel_scores, void *o_out, int32_t o_dtype, float *lse_out,
                                     void *ws_dense, size_t ws_dense_bytes, void *ws_sparse, size_t ws_sparse_bytes,
                                     void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (o_dtype != HGCA_F32 && o_dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, window, true)) != HGCA_OK) return rc;
    if ((rc = check_view(shape, pool, true)) != HGCA_OK) return rc;
    if (!q || !aligned16(q) || !o_out || !aligned16(o_out) || !cnt || k_max < 0 || (k_max > 0 && !idx))
        return HGCA_ERR_INVALID_ARG;
    const WsLayout wd = layout(shape, window->cap, 0);
    const WsLayout wsp = layout(shape, k_max, 0);
    if (!ws_dense || ws_dense_bytes < wd.total || !aligned16(ws_dense)) return HGCA_ERR_WORKSPACE;
    if (!ws_sparse || ws_sparse_bytes < wsp.total || !aligned16(ws_sparse)) return HGCA_ERR_WORKSPACE;
    if (ws_dense == ws_sparse) return HGCA_ERR_WORKSPACE;       // the two parts are live at the same time
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    AttnArgs da{};
    da.sh = to_dev(shape);
    da.q = q;
    da.kv = to_dev(window);
    const bool one_launch = HGCA_FUSE_DENSE_GATHER && window->cap > 0 && k_max > 0 && pool->cap > 0 &&
                            dense_gather_fusable(shape->dtype, shape->head_dim, group_of(shape));
    da.chunk = dense_chunk(shape, window->cap, one_launch);
    da.part = partials_at(ws_dense, wd, n_splits_for(window->cap, da.chunk));
    AttnArgs ga{};
    ga.sh = da.sh;
    ga.q = q;
    ga.kv = to_dev(pool);
    ga.idx = idx;
    ga.cnt = cnt;
    ga.sel_scores = sel_scores;
    ga.k_max = k_max;
    ga.chunk = pick_chunk(k_max, (int64_t)shape->batch * shape->n_q_heads, HGCA_TARGET_WGS_SPARSE);
    ga.part = partials_at(ws_sparse, wsp, std::max(1, n_splits_for(k_max, ga.chunk)));
    // gpu_attention over the window and cpu_attention over the listed entries: one launch where the shapes allow
    if (one_launch) {
        if ((rc = from_hip(launch_dense_gather(shape->dtype, shape->head_dim, da, ga, s))) != HGCA_OK) return rc;
    } else {
        if ((rc = from_hip(launch_attn_partial_dense(shape->dtype, shape->head_dim, da, s))) != HGCA_OK) return rc;
        if ((rc = from_hip(launch_attn_partial_gather(shape->dtype, shape->head_dim, ga, s))) != HGCA_OK) return rc;
    }
    // merge_state over all split partials of both parts
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_combine2(shape->head_dim, rows, da.part, ga.part, o_out, o_dtype, lse_out, s));
}

int hgca_lse_merge(const hgca_shape *shape, const float *o_a, const float *lse_a, const float *o_b,
                   const float *lse_b, void *o_out, int32_t o_dtype, float *lse_out, void *hip_stream)
{
    if (!shape || shape->batch < 0 || shape->n_q_heads <= 0) return HGCA_ERR_INVALID_ARG;
    if (shape->head_dim != 64 && shape->head_dim != 128) return HGCA_ERR_UNSUPPORTED;
    if (o_dtype != HGCA_F32 && o_dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (shape->batch == 0) return HGCA_OK;
    if (!o_a || !lse_a || !o_b || !lse_b || !o_out) return HGCA_ERR_INVALID_ARG;
    if (o_dtype == HGCA_BF16 && (o_out == (const void *)o_a || o_out == (const void *)o_b))
        return HGCA_ERR_INVALID_ARG;             // a bf16 result cannot overwrite an fp32 input in place
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    return from_hip(launch_merge(shape->head_dim, rows, o_a, lse_a, o_b, lse_b, o_out, o_dtype, lse_out,
                                 static_cast<hipStream_t>(hip_stream)));
}

namespace {

int check_cache(const hgca_shape *shape, const hgca_cache_state *c, CacheDev *out)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (!c) return HGCA_ERR_INVALID_ARG;
    if (c->block_size <= 0 || c->max_blocks <= 0 || c->win_blocks <= 0 || c->win_blocks > c->max_blocks || c->k_max < 0 ||
        c->pool_cap < 0)
        return HGCA_ERR_INVALID_ARG;
    if (c->block_size % 16 != 0) return HGCA_ERR_UNSUPPORTED;
    if (c->win_cap_blocks != 0 && (c->win_cap_blocks < c->win_blocks || c->win_cap_blocks > c->max_blocks))
        return HGCA_ERR_INVALID_ARG;
    if (shape->batch > 0 &&
        (!c->k_blocks || !c->v_blocks || !aligned16(c->k_blocks) || !aligned16(c->v_blocks) || !c->block_table ||
         !c->first_win_block || !c->win_lens || !c->pool_lens || !c->a_maw || !c->ctx_cnt || !c->plan || !c->status ||
         (c->k_max > 0 && !c->ctx_idx)))
        return HGCA_ERR_INVALID_ARG;
    out->k_blocks = static_cast<char *>(c->k_blocks);
    out->v_blocks = static_cast<char *>(c->v_blocks);
    out->block_table = c->block_table;
    out->first_win_block = c->first_win_block;
    out->win_lens = c->win_lens;
    out->pool_lens = c->pool_lens;
    out->a_maw = c->a_maw;
    out->ctx_idx = c->ctx_idx;
    out->ctx_cnt = c->ctx_cnt;
    out->plan = c->plan;
    out->status = c->status;
    out->a_evicted = c->a_evicted;
    out->block_size = c->block_size;
    out->max_blocks = c->max_blocks;
    out->win_blocks = c->win_blocks;
    out->k_max = c->k_max;
    out->pool_cap = c->pool_cap;
    out->win_cap = (c->win_cap_blocks ? c->win_cap_blocks : c->win_blocks) * c->block_size;
    return HGCA_OK;
}

}  // namespace

int hgca_kv_append_tokens(const hgca_shape *shape, const hgca_cache_state *cache, const void *k_in, const void *v_in,
                          int32_t n_tokens, const int32_t *active, void *hip_stream)
{
    CacheDev c{};
    int rc = check_cache(shape, cache, &c);
    if (rc != HGCA_OK) return rc;
    if (n_tokens < 0) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0 || n_tokens == 0) return HGCA_OK;
    if (!k_in || !v_in || !aligned16(k_in) || !aligned16(v_in)) return HGCA_ERR_INVALID_ARG;
    const int32_t row_bytes = shape->head_dim * (shape->dtype == HGCA_BF16 ? 2 : 4);
    return from_hip(launch_kv_append(c, k_in, v_in, active, shape->batch, shape->n_kv_heads, row_bytes, n_tokens,
                                     static_cast<hipStream_t>(hip_stream)));
}

int hgca_kv_append(const hgca_shape *shape, const hgca_cache_state *cache, const void *k_in, const void *v_in,
                   const int32_t *active, void *hip_stream)
{
    return hgca_kv_append_tokens(shape, cache, k_in, v_in, 1, active, hip_stream);
}

int hgca_kv_evict(const hgca_shape *shape, const hgca_cache_state *cache, double beta, void *hip_stream)
{
    CacheDev c{};
    int rc = check_cache(shape, cache, &c);
    if (rc != HGCA_OK) return rc;
    if (!(beta >= 0.0)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0) return HGCA_OK;
    return from_hip(launch_kv_evict(c, shape->batch, shape->n_q_heads, beta, static_cast<hipStream_t>(hip_stream)));
}

int hgca_managed_decode_step(const hgca_shape *shape, const hgca_cache_state *cache, const void *q, const void *k_in,
                             const void *v_in, float alpha, double beta, float *a_gpu,
                             void *o_out, int32_t o_dtype, float *lse_out, void *ws_dense, size_t ws_dense_bytes,
                             void *ws_sparse, size_t ws_sparse_bytes, void *hip_stream)
{
    CacheDev c{};
    int rc = check_cache(shape, cache, &c);
    if (rc != HGCA_OK) return rc;
    if (o_dtype != HGCA_F32 && o_dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;
    if (!(alpha >= 0.f && alpha <= 1.f) || !(beta >= 0.0)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0) return HGCA_OK;
    if (!q || !aligned16(q) || !k_in || !v_in || !aligned16(k_in) || !aligned16(v_in) || !a_gpu || !o_out ||
        !aligned16(o_out))
        return HGCA_ERR_INVALID_ARG;
    // the two tiers as ranges of the sequence's block list
    hgca_kv_view window{}, pool{};
    window.k = pool.k = cache->k_blocks;
    window.v = pool.v = cache->v_blocks;
    window.block_table = pool.block_table = cache->block_table;
    window.block_size = pool.block_size = cache->block_size;
    window.max_blocks = pool.max_blocks = cache->max_blocks;
    window.seq_lens = cache->win_lens;
    window.first_block = cache->first_win_block;
    window.cap = c.win_cap;
    pool.seq_lens = cache->pool_lens;
    pool.cap = cache->pool_cap;
    if ((rc = check_view(shape, &window, true)) != HGCA_OK) return rc;
    if ((rc = check_view(shape, &pool, true)) != HGCA_OK) return rc;
    const WsLayout wd = layout(shape, window.cap, 0);
    const WsLayout wsp = layout(shape, cache->k_max, 0);
    if (!ws_dense || ws_dense_bytes < wd.total || !aligned16(ws_dense)) return HGCA_ERR_WORKSPACE;
    if (!ws_sparse || ws_sparse_bytes < wsp.total || !aligned16(ws_sparse) || ws_sparse == ws_dense) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    const int32_t row_bytes = shape->head_dim * (shape->dtype == HGCA_BF16 ? 2 : 4);

    const bool one_launch = HGCA_FUSE_DENSE_GATHER && window.cap > 0 && cache->k_max > 0 && cache->pool_cap > 0 &&
                            dense_gather_fusable(shape->dtype, shape->head_dim, group_of(shape));
    // Alg. 2: KV_gpu' = concat(KV_gpu, KV_in): a launch of its own, or (token_joins_in_split) the window split that
    // owns the token's position writes its rows and the step's last launch stores the new length
    const bool token_joins_in_split = HGCA_FUSE_KV_APPEND && HGCA_FUSE_DECODE_TAIL && one_launch;
    if (!token_joins_in_split &&
        (rc = from_hip(launch_kv_append(c, k_in, v_in, nullptr, shape->batch, shape->n_kv_heads, row_bytes, 1, s))) != HGCA_OK)
        return rc;
    // gpu_attention: split kernels of the window, leaving the scaled scores in a_gpu
    AttnArgs da{};
    da.sh = to_dev(shape);
    da.q = q;
    da.kv = to_dev(&window);
    da.chunk = dense_chunk(shape, window.cap, one_launch);
    da.part = partials_at(ws_dense, wd, n_splits_for(window.cap, da.chunk));
    da.raw_scores = a_gpu;
    // cpu_attention over KV_ctx: split kernels over each head's list of salient pool positions
    AttnArgs ga{};
    ga.sh = da.sh;
    ga.q = q;
    ga.kv = to_dev(&pool);
    ga.idx = cache->ctx_idx;
    ga.cnt = cache->ctx_cnt;
    ga.k_max = cache->k_max;
    ga.chunk = pick_chunk(cache->k_max, rows, HGCA_TARGET_WGS_SPARSE);
    ga.part = partials_at(ws_sparse, wsp, std::max(1, n_splits_for(cache->k_max, ga.chunk)));
    // the two parts need nothing from each other: one launch where the shapes allow
    if (one_launch) {
        if ((rc = from_hip(launch_dense_gather(shape->dtype, shape->head_dim, da, ga, s, token_joins_in_split ? k_in : nullptr,
                                               token_joins_in_split ? v_in : nullptr))) != HGCA_OK)
            return rc;
    } else {
        if ((rc = from_hip(launch_attn_partial_dense(shape->dtype, shape->head_dim, da, s))) != HGCA_OK) return rc;
        if ((rc = from_hip(launch_attn_partial_gather(shape->dtype, shape->head_dim, ga, s))) != HGCA_OK) return rc;
    }
    // merge_state over all split partials; A_gpu = e^{s - lse_g} with the window's own lse from the same fold;
    // Alg. 1: A_maw <- (1 - alpha) A_maw + alpha A_gpu (the inserted token has no history); eviction and
    // sparsification where a window is full.  All three are per (sequence, head) row: one launch.
    if (HGCA_FUSE_DECODE_TAIL)
        return from_hip(launch_decode_tail(shape->head_dim, rows, da.part, ga.part, o_out, o_dtype, lse_out, a_gpu, c,
                                           shape->n_q_heads, alpha, beta, token_joins_in_split ? 1 : 0, s));
    float *lse_w = reinterpret_cast<float *>(static_cast<char *>(ws_dense) + wd.row_aux);
    if ((rc = from_hip(launch_combine2(shape->head_dim, rows, da.part, ga.part, o_out, o_dtype, lse_out, s, lse_w))) != HGCA_OK)
        return rc;
    if ((rc = from_hip(launch_window_weights(a_gpu, lse_w, window.seq_lens, rows, shape->n_q_heads, window.cap, c.a_maw, 1,
                                             alpha, s))) != HGCA_OK)
        return rc;
    return from_hip(launch_kv_evict(c, shape->batch, shape->n_q_heads, beta, s));
}

int hgca_ctx_compact(const hgca_shape *shape, const hgca_kv_view *pool, const int32_t *idx, const int32_t *cnt,
                     int32_t k_max, const int32_t *first_row, void *k_ctx, void *v_ctx, int32_t ctx_cap,
                     int32_t *cnt_out, void *hip_stream)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (k_max < 0 || ctx_cap < 0) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0) return HGCA_OK;
    if ((rc = check_view(shape, pool, true)) != HGCA_OK) return rc;
    if (!cnt || (k_max > 0 && !idx)) return HGCA_ERR_INVALID_ARG;
    if (ctx_cap > 0 && (!k_ctx || !v_ctx || !aligned16(k_ctx) || !aligned16(v_ctx) || k_ctx == v_ctx))
        return HGCA_ERR_INVALID_ARG;
    if (cnt_out && (cnt_out == first_row || cnt_out == cnt)) return HGCA_ERR_INVALID_ARG;   // read by other workgroups
    CtxCompactArgs a{};
    a.sh = to_dev(shape);
    a.kv = to_dev(pool);
    a.idx = idx;
    a.cnt = cnt;
    a.first_row = first_row;
    a.cnt_out = cnt_out;
    a.k_ctx = static_cast<char *>(k_ctx);
    a.v_ctx = static_cast<char *>(v_ctx);
    a.k_max = k_max;
    a.ctx_cap = ctx_cap;
    a.row_bytes = shape->head_dim * (shape->dtype == HGCA_BF16 ? 2 : 4);
    return from_hip(launch_ctx_compact(a, static_cast<hipStream_t>(hip_stream)));
}

namespace {

// Split size of the append-stage attention: enough workgroups to fill the GPU, few enough splits that the
// per-row partials stay small beside the K/V traffic.
int append_want_splits(const hgca_shape *s, int32_t n_q)
{
    const int64_t n_qb = ((int64_t)n_q * group_of(s) + 127) / 128;
    const int64_t units = std::max<int64_t>(1, (int64_t)s->batch * s->n_kv_heads * n_qb);
    return (int)std::max<int64_t>(1, HGCA_APPEND_TARGET_WGS / units);
}

int append_chunk(const hgca_shape *s, int32_t n_q, int64_t cap)
{
    const int want = append_want_splits(s, n_q);
    int64_t chunk = (std::max<int64_t>(cap, 1) + want - 1) / want;
    chunk = (chunk + 63) / 64 * 64;
    return (int)std::min<int64_t>(kMaxAppendChunk, std::max<int64_t>(kMinChunk, chunk));
}

struct AppendWs {
    size_t o, m, l, total;
    int max_splits;
};

AppendWs append_layout(const hgca_shape *s, int32_t n_q, int64_t max_tokens)
{
    AppendWs w{};
    // bf16: splits of up to kMaxAppendChunk tokens; fp32 runs on the one-query kernels, whose splits hold kMaxChunk
    w.max_splits = std::max(append_want_splits(s, n_q), n_splits_for(std::max<int64_t>(max_tokens, 1),
                                                                     s->dtype == HGCA_F32 ? kMaxChunk : kMaxAppendChunk));
    const size_t rows = (size_t)s->batch * n_q * s->n_q_heads;
    size_t at = 0;
    w.o = at; at += align_up(rows * w.max_splits * s->head_dim * sizeof(float));
    w.m = at; at += align_up(rows * w.max_splits * sizeof(float));
    w.l = at; at += align_up(rows * w.max_splits * sizeof(float));
    w.total = std::max<size_t>(at, kAlign);
    return w;
}

int check_append(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *tier, bool need_v)
{
    int rc = check_shape(shape);
    if (rc != HGCA_OK) return rc;
    if (n_q < 0 || n_q > 4096) return HGCA_ERR_INVALID_ARG;
    // the kernels keep the running maximum on the raw scores and apply the scale inside the exponent
    if (!(shape->sm_scale > 0.f) || !(shape->sm_scale < 3.0e38f)) return HGCA_ERR_INVALID_ARG;
    if ((rc = check_view(shape, tier, need_v)) != HGCA_OK) return rc;
    if (shape->batch > 0 && n_q > 0 && (!q || !aligned16(q))) return HGCA_ERR_INVALID_ARG;
    return HGCA_OK;
}

}  // namespace

size_t hgca_append_workspace_bytes(const hgca_shape *shape, int32_t n_q, int32_t max_tokens)
{
    if (check_shape(shape) != HGCA_OK || n_q < 0 || max_tokens < 0) return 0;
    return append_layout(shape, n_q, max_tokens).total;
}

int hgca_append_attn(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *tier,
                     int32_t flags, float *o_out, float *lse_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_append(shape, q, n_q, tier, true);
    if (rc != HGCA_OK) return rc;
    if (flags & ~(HGCA_APPEND_CAUSAL_TAIL | HGCA_APPEND_ONE_PART_P)) return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0 || n_q == 0) return HGCA_OK;
    if (!o_out || !lse_out || !aligned16(o_out)) return HGCA_ERR_INVALID_ARG;
    // (KV head, block of 128 query rows) pairs are one grid dimension of the launch
    if ((int64_t)shape->n_kv_heads * (((int64_t)n_q * group_of(shape) + 127) / 128) > 65535) return HGCA_ERR_UNSUPPORTED;
    const AppendWs w = append_layout(shape, n_q, tier->cap);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    if (shape->dtype == HGCA_F32) {
        // fp32 inputs: every (sequence, query) pair is a one-query attention over the tokens that query sees, so the
        // split kernels of the decode path serve, on a batch of B * n_q queries that share their sequence's rows
        if ((int64_t)shape->batch * n_q > 65535) return HGCA_ERR_UNSUPPORTED;
        AttnArgs d{};
        d.sh = to_dev(shape);
        d.sh.batch = shape->batch * n_q;
        d.q = q;
        d.kv = to_dev(tier);
        d.kv.n_q = n_q;
        d.kv.causal_tail = (flags & HGCA_APPEND_CAUSAL_TAIL) ? 1 : 0;
        d.chunk = pick_chunk(tier->cap, (int64_t)d.sh.batch * shape->n_kv_heads, HGCA_TARGET_WGS_DENSE);
        char *base = static_cast<char *>(ws);
        d.part.o = reinterpret_cast<float *>(base + w.o);
        d.part.m = reinterpret_cast<float *>(base + w.m);
        d.part.l = reinterpret_cast<float *>(base + w.l);
        d.part.n_splits = std::max(1, n_splits_for(tier->cap, d.chunk));
        if (d.part.n_splits > w.max_splits) return HGCA_ERR_WORKSPACE;
        const int64_t rows = (int64_t)d.sh.batch * shape->n_q_heads;
        if (tier->cap == 0) {                    // nothing to attend to: the fold of one empty split writes O = 0, lse = -inf
            Partials none{};
            return from_hip(launch_combine2(shape->head_dim, rows, none, none, o_out, 0, lse_out, s));
        }
        if ((rc = from_hip(launch_attn_partial_dense(shape->dtype, shape->head_dim, d, s))) != HGCA_OK) return rc;
        return from_hip(launch_combine(shape->head_dim, rows, d.part, o_out, lse_out, s));
    }
    AppendArgs a{};
    a.sh = to_dev(shape);
    a.q = q;
    a.kv = to_dev(tier);
    a.n_q = n_q;
    a.causal_tail = (flags & HGCA_APPEND_CAUSAL_TAIL) ? 1 : 0;
    a.one_part_p = (flags & HGCA_APPEND_ONE_PART_P) ? 1 : 0;
    a.chunk = append_chunk(shape, n_q, tier->cap);
    char *base = static_cast<char *>(ws);
    a.part.o = reinterpret_cast<float *>(base + w.o);
    a.part.m = reinterpret_cast<float *>(base + w.m);
    a.part.l = reinterpret_cast<float *>(base + w.l);
    a.part.n_splits = std::max(1, n_splits_for(tier->cap, a.chunk));
    if (a.part.n_splits > w.max_splits) return HGCA_ERR_WORKSPACE;
    if ((rc = from_hip(launch_append_attn(shape->head_dim, a, s))) != HGCA_OK) return rc;
    const int64_t rows = (int64_t)shape->batch * n_q * shape->n_q_heads;
    return from_hip(launch_combine(shape->head_dim, rows, a.part, o_out, lse_out, s));
}

namespace {

// Workspace of the two-tier append attention: split partials of the window and of the pool (the split counts are
// chosen for the two tiers together), and the two per-tier lse rows for callers that do not ask for them.
struct TiersWs {
    size_t o_w, m_w, l_w, o_p, m_p, l_p, lse_w, lse_p, total;
    int chunk_w, chunk_p, n_w, n_p;
};

TiersWs tiers_layout(const hgca_shape *s, int32_t n_q, int64_t win_cap, int64_t pool_cap)
{
    TiersWs w{};
    // The splits of a unit are shared out between the tiers in proportion to their capacities (each tier that has
    // any capacity gets at least one), so that the launch has about as many workgroups as the device holds at once;
    // a tier whose share would make its splits longer than kMaxAppendChunk gets more.  The kernel then shares a
    // tier's ACTUAL length out evenly among its splits (the capacity only bounds it).
    const int want = append_want_splits(s, n_q);
    const int64_t total = win_cap + pool_cap;
    auto splits = [&](int64_t cap, int64_t other) -> int {
        if (cap <= 0) return 0;
        int64_t n = other > 0 ? std::max<int64_t>(1, std::min<int64_t>(want - 1, (cap * want + total / 2) / total)) : want;
        n = std::max<int64_t>(n, (cap + kMaxAppendChunk - 1) / kMaxAppendChunk);
        return (int)std::min<int64_t>(n, (cap + kMinChunk - 1) / kMinChunk);
    };
    auto chunk_of = [](int64_t cap, int n) -> int {
        if (n == 0) return kMinChunk;
        return (int)std::max<int64_t>(kMinChunk, ((cap + n - 1) / n + 63) / 64 * 64);
    };
    w.n_w = splits(win_cap, pool_cap);
    w.n_p = pool_cap > 0 ? (win_cap > 0 ? std::max(1, std::max(want - w.n_w, 1)) : want) : 0;
    if (pool_cap > 0) {
        w.n_p = (int)std::max<int64_t>(w.n_p, (pool_cap + kMaxAppendChunk - 1) / kMaxAppendChunk);
        w.n_p = (int)std::min<int64_t>(w.n_p, (pool_cap + kMinChunk - 1) / kMinChunk);
    }
    w.chunk_w = chunk_of(win_cap, w.n_w);
    w.chunk_p = chunk_of(pool_cap, w.n_p);
    w.n_w = win_cap > 0 ? n_splits_for(win_cap, w.chunk_w) : 0;
    w.n_p = pool_cap > 0 ? n_splits_for(pool_cap, w.chunk_p) : 0;
    const size_t rows = (size_t)s->batch * n_q * s->n_q_heads;
    size_t at = 0;
    w.o_w = at; at += align_up(rows * w.n_w * s->head_dim * sizeof(float));
    w.m_w = at; at += align_up(rows * w.n_w * sizeof(float));
    w.l_w = at; at += align_up(rows * w.n_w * sizeof(float));
    w.o_p = at; at += align_up(rows * w.n_p * s->head_dim * sizeof(float));
    w.m_p = at; at += align_up(rows * w.n_p * sizeof(float));
    w.l_p = at; at += align_up(rows * w.n_p * sizeof(float));
    w.lse_w = at; at += align_up(rows * sizeof(float));
    w.lse_p = at; at += align_up(rows * sizeof(float));
    w.total = std::max<size_t>(at, kAlign);
    return w;
}

}  // namespace

size_t hgca_append_tiers_workspace_bytes(const hgca_shape *shape, int32_t n_q, int32_t window_cap, int32_t pool_cap)
{
    if (check_shape(shape) != HGCA_OK || n_q < 0 || window_cap < 0 || pool_cap < 0) return 0;
    return tiers_layout(shape, n_q, window_cap, pool_cap).total;
}

int hgca_append_attn_tiers(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *window,
                           const hgca_kv_view *pool, int32_t flags, float *o_out, float *lse_out, float *lse_window_out,
                           float *lse_pool_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_append(shape, q, n_q, window, true);
    if (rc != HGCA_OK) return rc;
    if ((rc = check_append(shape, q, n_q, pool, true)) != HGCA_OK) return rc;
    if (flags & ~(HGCA_APPEND_CAUSAL_TAIL | HGCA_APPEND_ONE_PART_P)) return HGCA_ERR_INVALID_ARG;
    if (shape->dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;      // fp32 inputs: one call per tier and hgca_lse_merge
    if (shape->batch == 0 || n_q == 0) return HGCA_OK;
    if (!o_out || !lse_out || !aligned16(o_out)) return HGCA_ERR_INVALID_ARG;
    if ((int64_t)shape->n_kv_heads * (((int64_t)n_q * group_of(shape) + 127) / 128) > 65535) return HGCA_ERR_UNSUPPORTED;
    const TiersWs w = tiers_layout(shape, n_q, window->cap, pool->cap);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);

    AppendArgs aw{}, ap{};
    aw.sh = ap.sh = to_dev(shape);
    aw.q = ap.q = q;
    aw.n_q = ap.n_q = n_q;
    aw.one_part_p = ap.one_part_p = (flags & HGCA_APPEND_ONE_PART_P) ? 1 : 0;
    aw.chunk = w.chunk_w;
    ap.chunk = w.chunk_p;
    aw.kv = to_dev(window);
    aw.causal_tail = (flags & HGCA_APPEND_CAUSAL_TAIL) ? 1 : 0;
    aw.part = Partials{reinterpret_cast<float *>(base + w.o_w), reinterpret_cast<float *>(base + w.m_w),
                       reinterpret_cast<float *>(base + w.l_w), w.n_w};
    ap.kv = to_dev(pool);
    ap.causal_tail = 0;
    ap.part = Partials{reinterpret_cast<float *>(base + w.o_p), reinterpret_cast<float *>(base + w.m_p),
                       reinterpret_cast<float *>(base + w.l_p), w.n_p};
    // the pool's splits take the lower block numbers: they are the bulk of the launch
    if ((rc = from_hip(launch_append_attn2(shape->head_dim, ap, aw, s))) != HGCA_OK) return rc;
    // merge_state over the splits of both tiers at once; each tier's own lse comes out of the same fold
    const int64_t rows = (int64_t)shape->batch * n_q * shape->n_q_heads;
    float *lse_w = lse_window_out ? lse_window_out : reinterpret_cast<float *>(base + w.lse_w);
    float *lse_p = lse_pool_out ? lse_pool_out : reinterpret_cast<float *>(base + w.lse_p);
    const bool want_tiers = lse_window_out || lse_pool_out;
    return from_hip(launch_combine2(shape->head_dim, rows, aw.part, ap.part, o_out, 0, lse_out, s,
                                    want_tiers ? lse_w : nullptr, want_tiers ? lse_p : nullptr));
}

namespace {

// Arguments of the weights pass over one tier (bf16) and the number of workgroups along x it takes.
int weights_args(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *tier, int32_t causal_tail,
                 const float *lse, float *a_out, AppendArgs *a)
{
    a->sh = to_dev(shape);
    a->q = q;
    a->kv = to_dev(tier);
    a->n_q = n_q;
    a->causal_tail = causal_tail ? 1 : 0;
    a->lse = lse;
    a->a_out = a_out;
    const int64_t units = (int64_t)shape->batch * shape->n_kv_heads;
    a->chunk = 2048;                                 // tokens per workgroup, halved until the GPU is filled
    while (a->chunk > 64 && units * n_splits_for(tier->cap, a->chunk) < HGCA_WEIGHTS_TARGET_WGS) a->chunk /= 2;
    return tier->cap > 0 ? n_splits_for(tier->cap, a->chunk) : 0;
}

}  // namespace

int hgca_append_weights_tiers(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *window,
                              const hgca_kv_view *pool, int32_t causal_tail, const float *lse_window, const float *lse_pool,
                              float *a_gpu, float *a_cpu, void *hip_stream)
{
    int rc = check_append(shape, q, n_q, window, false);
    if (rc != HGCA_OK) return rc;
    if ((rc = check_append(shape, q, n_q, pool, false)) != HGCA_OK) return rc;
    if (n_q == 0) return HGCA_ERR_INVALID_ARG;       // an average over no query is undefined
    if (shape->dtype != HGCA_BF16) return HGCA_ERR_UNSUPPORTED;      // fp32 inputs: one call per tier
    if (shape->batch == 0) return HGCA_OK;
    if ((window->cap > 0 && (!lse_window || !a_gpu)) || (pool->cap > 0 && (!lse_pool || !a_cpu))) return HGCA_ERR_INVALID_ARG;
    AppendArgs aw{}, ap{};
    const int n_w = weights_args(shape, q, n_q, window, causal_tail, lse_window, a_gpu, &aw);
    const int n_p = weights_args(shape, q, n_q, pool, 0, lse_pool, a_cpu, &ap);
    // the pool's workgroups take the lower block numbers: they are the bulk of the launch
    return from_hip(launch_append_weights2(shape->head_dim, ap, n_p, aw, n_w, static_cast<hipStream_t>(hip_stream)));
}

int hgca_append_weights(const hgca_shape *shape, const void *q, int32_t n_q, const hgca_kv_view *tier,
                        int32_t causal_tail, const float *lse, float *a_out, void *hip_stream)
{
    int rc = check_append(shape, q, n_q, tier, false);
    if (rc != HGCA_OK) return rc;
    if (n_q == 0) return HGCA_ERR_INVALID_ARG;       // an average over no query is undefined
    if (shape->batch == 0 || tier->cap == 0) return HGCA_OK;
    if (!lse || !a_out) return HGCA_ERR_INVALID_ARG;
    AppendArgs a{};
    const int n_chunks = weights_args(shape, q, n_q, tier, causal_tail, lse, a_out, &a);
    if (shape->dtype == HGCA_F32)
        return from_hip(launch_append_weights_f32(shape->head_dim, a, static_cast<hipStream_t>(hip_stream)));
    return from_hip(launch_append_weights(shape->head_dim, a, n_chunks, static_cast<hipStream_t>(hip_stream)));
}

namespace {

// Workspace of hgca_managed_append_step: [scratch of hgca_append_attn | O, lse of the window part | O, lse of the pool part]
struct ManagedAppendWs {
    size_t attn, o_w, lse_w, o_p, lse_p, total;
    size_t attn_bytes;
};

ManagedAppendWs managed_append_layout(const hgca_shape *s, int32_t n_q, int32_t win_cap, int32_t pool_cap)
{
    ManagedAppendWs w{};
    const size_t rows = (size_t)s->batch * n_q * s->n_q_heads;
    w.attn_bytes = std::max(append_layout(s, n_q, std::max(win_cap, pool_cap)).total,
                            tiers_layout(s, n_q, win_cap, pool_cap).total);
    size_t at = 0;
    w.attn = at; at += align_up(w.attn_bytes);
    w.o_w = at; at += align_up(rows * s->head_dim * sizeof(float));
    w.lse_w = at; at += align_up(rows * sizeof(float));
    w.o_p = at; at += align_up(rows * s->head_dim * sizeof(float));
    w.lse_p = at; at += align_up(rows * sizeof(float));
    w.total = std::max<size_t>(at, kAlign);
    return w;
}

}  // namespace

size_t hgca_managed_append_workspace_bytes(const hgca_shape *shape, const hgca_cache_state *cache, int32_t n_q)
{
    CacheDev c{};
    hgca_shape host_only = shape ? *shape : hgca_shape{};
    host_only.batch = shape ? std::min(shape->batch, 0) : 0;     // sizing needs no device pointers
    if (!shape || !cache || n_q < 0 || n_q > 4096 || check_shape(shape) != HGCA_OK || check_cache(&host_only, cache, &c) != HGCA_OK)
        return 0;
    return managed_append_layout(shape, n_q, c.win_cap, c.pool_cap).total;
}

int hgca_managed_append_step(const hgca_shape *shape, const hgca_cache_state *cache, const void *q, const void *k_in,
                             const void *v_in, int32_t n_q, float alpha, double beta, int32_t flags, float *a_gpu,
                             float *a_cpu, float *o_out, float *lse_out, void *ws, size_t ws_bytes, void *hip_stream)
{
    CacheDev c{};
    int rc = check_cache(shape, cache, &c);
    if (rc != HGCA_OK) return rc;
    if (n_q < 0 || n_q > 4096 || !(alpha >= 0.f && alpha <= 1.f) || !(beta >= 0.0) || (flags & ~HGCA_APPEND_ONE_PART_P))
        return HGCA_ERR_INVALID_ARG;
    if (shape->batch == 0 || n_q == 0) return HGCA_OK;
    // the two tiers as ranges of the sequence's block list
    hgca_kv_view window{}, pool{};
    window.k = pool.k = cache->k_blocks;
    window.v = pool.v = cache->v_blocks;
    window.block_table = pool.block_table = cache->block_table;
    window.block_size = pool.block_size = cache->block_size;
    window.max_blocks = pool.max_blocks = cache->max_blocks;
    window.seq_lens = cache->win_lens;
    window.first_block = cache->first_win_block;
    window.cap = c.win_cap;
    pool.seq_lens = cache->pool_lens;
    pool.cap = cache->pool_cap;
    if ((rc = check_append(shape, q, n_q, &window, true)) != HGCA_OK) return rc;
    if ((rc = check_append(shape, q, n_q, &pool, true)) != HGCA_OK) return rc;
    if ((int64_t)shape->batch * n_q > 65535) return HGCA_ERR_UNSUPPORTED;        // the merge runs on batch * n_q rows
    if (!k_in || !v_in || !aligned16(k_in) || !aligned16(v_in) || !a_gpu || (cache->pool_cap > 0 && !a_cpu) || !o_out ||
        !lse_out || !aligned16(o_out))
        return HGCA_ERR_INVALID_ARG;
    const ManagedAppendWs w = managed_append_layout(shape, n_q, c.win_cap, c.pool_cap);
    if (!ws || ws_bytes < w.total || !aligned16(ws)) return HGCA_ERR_WORKSPACE;
    char *base = static_cast<char *>(ws);
    float *o_w = reinterpret_cast<float *>(base + w.o_w), *lse_w = reinterpret_cast<float *>(base + w.lse_w);
    float *o_p = reinterpret_cast<float *>(base + w.o_p), *lse_p = reinterpret_cast<float *>(base + w.lse_p);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int32_t row_bytes = shape->head_dim * (shape->dtype == HGCA_BF16 ? 2 : 4);

    // Alg. 2, append branch: KV_gpu' = concat(KV_gpu, KV_in)
    if ((rc = from_hip(launch_kv_append(c, k_in, v_in, nullptr, shape->batch, shape->n_kv_heads, row_bytes, n_q, s))) != HGCA_OK)
        return rc;
    // gpu_attention over the window (causal among the incoming tokens), cpu_attention over the complete offloaded
    // cache, merge_state per (sequence, query, head): bf16 as one launch for both tiers and one fold; fp32 as a call
    // per tier and a merge
    if (shape->dtype == HGCA_BF16) {
        if ((rc = hgca_append_attn_tiers(shape, q, n_q, &window, &pool, flags | HGCA_APPEND_CAUSAL_TAIL, o_out, lse_out,
                                         lse_w, lse_p, base + w.attn, w.attn_bytes, hip_stream)) != HGCA_OK)
            return rc;
    } else {
        if ((rc = hgca_append_attn(shape, q, n_q, &window, flags | HGCA_APPEND_CAUSAL_TAIL, o_w, lse_w, base + w.attn,
                                   w.attn_bytes, hip_stream)) != HGCA_OK)
            return rc;
        if ((rc = hgca_append_attn(shape, q, n_q, &pool, flags, o_p, lse_p, base + w.attn, w.attn_bytes, hip_stream)) != HGCA_OK)
            return rc;
        hgca_shape merged = *shape;
        merged.batch = shape->batch * n_q;
        if ((rc = hgca_lse_merge(&merged, o_p, lse_p, o_w, lse_w, o_out, HGCA_F32, lse_out, hip_stream)) != HGCA_OK) return rc;
    }
    // A_gpu, A_cpu: the query-averaged weights of the two parts (bf16: one launch for both)
    if (shape->dtype == HGCA_BF16) {
        if ((rc = hgca_append_weights_tiers(shape, q, n_q, &window, &pool, 1, lse_w, lse_p, a_gpu, a_cpu, hip_stream)) != HGCA_OK)
            return rc;
    } else {
        if ((rc = hgca_append_weights(shape, q, n_q, &window, 1, lse_w, a_gpu, hip_stream)) != HGCA_OK) return rc;
        if ((rc = hgca_append_weights(shape, q, n_q, &pool, 0, lse_p, a_cpu, hip_stream)) != HGCA_OK) return rc;
    }
    // Alg. 1: moving averages (the n_q new entries take their first observed weight), re-evaluation of the salient
    // lists (Sec. 3.2.2: ids = A_cpu > beta / A_cpu.size), eviction of as many whole blocks as it takes: per row, one launch
    if (HGCA_FUSE_APPEND_TAIL)
        return from_hip(launch_append_tail(c, a_gpu, cache->pool_cap > 0 ? a_cpu : nullptr, shape->batch, shape->n_q_heads,
                                           n_q, alpha, beta, s));
    const int64_t rows = (int64_t)shape->batch * shape->n_q_heads;
    if ((rc = from_hip(launch_maw_update(c.a_maw, a_gpu, c.win_lens, rows, shape->n_q_heads, c.win_cap, n_q, alpha, s))) != HGCA_OK)
        return rc;
    // re-evaluation (Sec. 3.2.2): the salient lists are replaced by ids = A_cpu > beta / A_cpu.size
    if (cache->pool_cap > 0) {
        ThresholdArgs t{};
        t.w = a_cpu;
        t.seq_lens = c.pool_lens;
        t.sizes = c.pool_lens;
        t.beta = beta;
        t.n_q_heads = shape->n_q_heads;
        t.cap = cache->pool_cap;
        t.k_max = c.k_max;
        t.idx = c.ctx_idx;
        t.cnt = c.ctx_cnt;
        t.status = c.status;
        t.status_bit = kCacheListFull;
        if ((rc = from_hip(launch_threshold_select(t, rows, s))) != HGCA_OK) return rc;
    }
    // eviction of as many whole blocks as it takes, sparsification of what leaves
    return from_hip(launch_kv_evict(c, shape->batch, shape->n_q_heads, beta, s));
}

}  // extern "C"
