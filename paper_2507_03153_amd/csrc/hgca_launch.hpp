// Host-side launch functions of the HGCA kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hgca_device.hpp"

namespace hgca {

constexpr int kMaxChunk = 512;     // tokens of one split (one workgroup) at most
constexpr int kMaxScoreChunk = 128;   // same for the MFMA score pass, which wants many small workgroups
constexpr int kMinChunk = 64;

// Split partials of softmax attention: for every (b, h, split)
//   m = max score, l = sum e^{s-m}, o[d] = sum e^{s-m} v   (not normalised).
struct Partials {
    float *o;      // [B*Hq, n_splits, d]
    float *m;      // [B*Hq, n_splits]
    float *l;      // [B*Hq, n_splits]
    int32_t n_splits;
};

struct AttnArgs {
    ShapeDev sh;
    const void *q;
    KvDev kv;
    const int32_t *idx;    // gather only: [B, Hq, k_max]
    const int32_t *cnt;    // gather only: [B, Hq]
    const float *sel_scores;   // gather only, optional: scaled scores of the listed entries (skips the K pass)
    int32_t k_max;
    int32_t chunk;         // tokens per split
    Partials part;
    float *raw_scores;     // dense only, optional: [B, Hq, cap], receives the scaled score of every valid token
    int32_t grouped;       // gather only: idx is [B, Hkv, k_max], cnt [B, Hkv]; the heads of a group share the list
};

// dtype: 0 fp32, 1 bf16; head_dim 64|128.  Dense handles the `group` query heads
// of one KV head per workgroup; gather handles one query head per workgroup.
hipError_t launch_attn_partial_dense(int dtype, int head_dim, const AttnArgs &a, hipStream_t s);
hipError_t launch_attn_partial_gather(int dtype, int head_dim, const AttnArgs &a, hipStream_t s);

hipError_t launch_combine(int head_dim, int64_t n_rows, const Partials &p, float *o, float *lse, hipStream_t s);
// Folds the splits of two partial sets (either may have n_splits == 0) into one result; o_dtype 0 fp32, 1 bf16.
hipError_t launch_combine2(int head_dim, int64_t n_rows, const Partials &p, const Partials &q, void *o, int o_dtype,
                           float *lse, hipStream_t s, float *lse_p = nullptr,   // lse_p / lse_q: optional lse of set p / q alone
                           float *lse_q = nullptr);

hipError_t launch_merge(int head_dim, int64_t n_rows, const float *o_a, const float *lse_a, const float *o_b,
                        const float *lse_b, void *o_out, int o_dtype, float *lse_out, hipStream_t s);

struct ScoreArgs {
    ShapeDev sh;
    const void *q;
    KvDev kv;
    float *scores;         // [B, Hq, cap] fp32, or [B, Hkv, cap] with group_max
    int32_t chunk;
    int32_t n_chunks;
    int32_t group_max;     // write the maximum over the heads of each group instead of every head's score
};
hipError_t launch_scores(int dtype, int head_dim, const ScoreArgs &a, hipStream_t s);

struct SelectArgs {
    ShapeDev sh;
    KvDev kv;              // only seq_lens / cap are used
    const float *scores;   // [B, Hq, cap]
    const int32_t *k_per_seq;
    int32_t k_uniform, k_max;
    int32_t *idx;          // [B, Hq, k_max]
    int32_t *cnt;          // [B, Hq]
    float *sel_scores;     // optional [B, Hq, k_max]: score of every kept entry, in idx order
};
hipError_t launch_select(const SelectArgs &a, hipStream_t s);

// The window's split kernels and the per-head gather's split kernels (launch_attn_partial_dense and
// launch_attn_partial_gather with the same arguments) as one launch; bf16, groups of 1, 2 or 4, per-head lists.
bool dense_gather_fusable(int dtype, int head_dim, int group);
// With k_new / v_new ([B, Hkv, row], paged window with a per-sequence first block only) the window takes one more
// token per sequence in the same launch: the split that owns its position writes its rows into the window's block
// first; the stored length is NOT updated (pending_window_len gives the length the launch works with).
hipError_t launch_dense_gather(int dtype, int head_dim, const AttnArgs &dense, const AttnArgs &gather, hipStream_t s,
                               const void *k_new = nullptr, const void *v_new = nullptr);

// Union of the index lists of the heads of each group: idx [B, Hq, k_max] / cnt [B, Hq] -> out [B, Hkv, k_max_out]
// ascending, -1 padded, out_cnt [B, Hkv].  Positions must lie in [0, n_positions).
hipError_t launch_union_lists(const int32_t *idx, const int32_t *cnt, int32_t k_max, int32_t batch, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t n_positions, int32_t *out, int32_t *out_cnt,
                              int32_t k_max_out, int32_t *status, hipStream_t s);

// ---- attention weights, their moving average, threshold rule ----

// a [n_rows, cap] holds scaled scores on entry and softmax weights e^{s - lse} on exit (0 beyond the length);
// maw (optional, [n_rows, cap]) receives the moving-average update with those weights in the same pass.
hipError_t launch_window_weights(float *a, const float *lse, const int32_t *seq_lens, int64_t n_rows, int32_t n_q_heads,
                                 int32_t cap, float *maw, int32_t n_new, float alpha, hipStream_t s);

hipError_t launch_maw_update(float *maw, const float *a_gpu, const int32_t *seq_lens, int64_t n_rows, int32_t n_q_heads,
                             int32_t cap, int32_t n_new, float alpha, hipStream_t s);

struct ThresholdArgs {
    const float *w;            // [B*Hq, cap]
    const int32_t *seq_lens;   // [B] or null
    const int32_t *sizes;      // [B] or null
    double beta;
    int32_t size_uniform, n_q_heads, cap, k_max;
    int32_t *idx;              // [B*Hq, k_max]
    int32_t *cnt;              // [B*Hq]
    float *w_norm;             // optional [B*Hq, k_max]
    int32_t *status;           // optional: receives status_bit (atomic or) when a row has more than k_max passing entries
    int32_t status_bit;
};
hipError_t launch_threshold_select(const ThresholdArgs &a, int64_t n_rows, hipStream_t s);

// ---- append stage: N queries per sequence over one tier (bf16, MFMA) ----

constexpr int kMaxAppendChunk = 8192;   // tokens of one split of the append-stage attention at most

struct AppendArgs {
    ShapeDev sh;
    const void *q;             // [B, N, Hq, d] bf16
    KvDev kv;
    int32_t n_q;               // N
    int32_t causal_tail;       // 1: the tier's last N valid tokens are the queries' own; query i sees tokens < len-N+i+1
    int32_t one_part_p;        // 1: the weights enter the second product as one bf16 value instead of a high and a low part
    int32_t chunk;             // tokens per split (attention) or per workgroup (weights), a multiple of 64
    Partials part;             // attention: rows are (b, query, head)
    const float *lse;          // weights: [B, N, Hq], the tier's log-sum-exp per query and head
    float *a_out;              // weights: [B, Hq, cap]
};
hipError_t launch_append_attn(int head_dim, const AppendArgs &a, hipStream_t s);
// two tiers in one launch (same queries and shape; each tier with its own view, mask rule, split size and partials)
hipError_t launch_append_attn2(int head_dim, const AppendArgs &a, const AppendArgs &a2, hipStream_t s);
hipError_t launch_append_weights(int head_dim, const AppendArgs &a, int n_chunks, hipStream_t s);
// the weights of two tiers (same queries and shape) in one launch
hipError_t launch_append_weights2(int head_dim, const AppendArgs &a, int n_chunks, const AppendArgs &a2, int n_chunks2,
                                  hipStream_t s);
// the same for fp32 inputs (q [B, N, Hq, d] fp32, fp32 tier): VALU pass, 64 tokens per workgroup
hipError_t launch_append_weights_f32(int head_dim, const AppendArgs &a, hipStream_t s);

// ---- KV manager over a block pool (mirrors hgca_cache_state; all pointers device memory) ----

constexpr int32_t kCacheWindowFull = 1, kCacheContextFull = 2, kCacheListFull = 4;   // sticky bits of *status

// Length of a window that takes n_new tokens: len + n_new if they fit the window's capacity and the sequence's table
// row; otherwise the window takes none of them, the stored length stands and *fail_bits (if given) names the reason.
// Every kernel that has to agree on the outcome before the new length is stored applies this one rule.
__device__ __forceinline__ int pending_window_len(int len, int first_block, int n_new, int cap, int block_size,
                                                  int max_blocks, int32_t *fail_bits)
{
    const bool no_room = len + n_new > cap;
    if (len < 0 || no_room || first_block + (len + n_new - 1) / block_size >= max_blocks) {
        if (fail_bits) *fail_bits = no_room ? kCacheWindowFull : kCacheContextFull;
        return len;
    }
    return len + n_new;
}

struct CacheDev {
    char *k_blocks, *v_blocks;
    const int32_t *block_table;
    int32_t *first_win_block, *win_lens, *pool_lens;
    float *a_maw;
    int32_t *ctx_idx, *ctx_cnt, *plan, *status;
    float *a_evicted;          // optional [B*Hq, pool_cap]
    int32_t block_size, max_blocks, win_blocks, k_max, pool_cap;
    int32_t win_cap;           // tokens the window may hold (>= win_blocks * block_size = l_max); row length of a_maw
};

// k_in / v_in: [B, n_tokens, Hkv, row]
hipError_t launch_kv_append(const CacheDev &c, const void *k_in, const void *v_in, const int32_t *active, int32_t batch,
                            int32_t n_kv_heads, int32_t row_bytes, int32_t n_tokens, hipStream_t s);
hipError_t launch_kv_evict(const CacheDev &c, int32_t batch, int32_t n_q_heads, double beta, hipStream_t s);
// Tail of an append turn: moving average with a_gpu (n_new new entries), salient lists replaced from a_cpu (may be
// null when the cache has no pool capacity), eviction and sparsification: one launch, one workgroup per row.
hipError_t launch_append_tail(const CacheDev &c, const float *a_gpu, const float *a_cpu, int32_t batch, int32_t n_q_heads,
                              int32_t n_new, float alpha, double beta, hipStream_t s);
// Fold of the window's (p) and the salient list's (q) split partials, window weights e^{s - lse_window} in place in
// a_gpu [n_rows, win_cap] with Alg. 1's moving average (one new token), eviction and sparsification: one launch.
// token_pending: the token's rows are in the window but the stored length does not count it yet (see
// launch_dense_gather); the launch then stores the new length, or raises the status bit if the token did not fit.
hipError_t launch_decode_tail(int head_dim, int64_t n_rows, const Partials &p, const Partials &q, void *o, int o_dtype,
                              float *lse, float *a_gpu, const CacheDev &c, int32_t n_q_heads, float alpha, double beta,
                              int32_t token_pending, hipStream_t s);

// Copy of listed pool entries into per-head contiguous storage (KV_ctx of Alg. 1).
struct CtxCompactArgs {
    ShapeDev sh;
    KvDev kv;                  // the pool
    const int32_t *idx, *cnt;  // [B*Hq, k_max], [B*Hq]
    const int32_t *first_row;  // optional [B*Hq]: rows of KV_ctx already taken
    int32_t *cnt_out;          // optional [B*Hq]: rows taken afterwards
    char *k_ctx, *v_ctx;       // [B*Hq, ctx_cap, row_bytes]
    int32_t k_max, ctx_cap, row_bytes;
};
hipError_t launch_ctx_compact(const CtxCompactArgs &a, hipStream_t s);

}  // namespace hgca
