// KV manager (Alg. 1) for tiers that live in one block pool in HBM: a sequence's KV entries sit in
// fixed-size blocks listed, in arrival order, in one row of a block table; the older pool is the
// first `first_win_block` blocks of the row and the recent window the blocks after them.  Inserting
// a token writes one K and one V row; evicting the oldest window block moves the boundary: no KV row
// is copied.  What does move is the per-entry moving average of attention weights, which is kept
// per window position: the evicted entries' averages are thresholded (Sec. 3.2.2) into the per-head
// lists of salient pool positions and the rest of the row shifts down.
#include <algorithm>

#include "hgca_launch.hpp"
#include "fold_device.hpp"
#include "row_map.hpp"
#include "threshold_compact.hpp"

namespace hgca {

namespace {

// The K and V rows of the n_tokens incoming tokens of every KV head go to the window positions len .. len + n_tokens
// - 1 (slot p % block_size of window block p / block_size); then the length grows.  A sequence whose window capacity
// or table row cannot take all of them receives none (status bit).  gridDim.y workgroups share a sequence's rows
// (16-byte pieces dealt round-robin, four loads in flight per thread); the last of them to finish (an arrival counter
// in plan[4b + 3], left at zero) stores the new length: by then every workgroup of the sequence has read the old one.
__global__ __launch_bounds__(kRowBlock) void kv_append_kernel(CacheDev c, const char *k_in, const char *v_in,
                                                              const int32_t *active, int32_t n_kv_heads,
                                                              int32_t row_bytes, int32_t n_tokens)
{
    const int b = blockIdx.x;
    if (active && !active[b]) return;
    const int len = c.win_lens[b];
    const int first = c.first_win_block[b];
    int32_t fail_bits = 0;
    if (pending_window_len(len, first, n_tokens, c.win_cap, c.block_size, c.max_blocks, &fail_bits) == len) {   // uniform
        if (threadIdx.x == 0 && blockIdx.y == 0) atomicOr(c.status, fail_bits);
        return;
    }
    const int pieces = row_bytes / 16;                         // 16-byte pieces of one row
    const int per_token = n_kv_heads * pieces;
    const int total = n_tokens * per_token, stride = kRowBlock * (int)gridDim.y;
    constexpr int U = 4;
    for (int i0 = (int)blockIdx.y * kRowBlock + (int)threadIdx.x; i0 < total; i0 += U * stride) {
        uint4 kr[U], vr[U];
        int64_t dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = min(i0 + u * stride, total - 1);
            const int t = i / per_token, kvh = (i % per_token) / pieces, p = i % pieces;
            const int pos = len + t;
            const int64_t blk = c.block_table[(int64_t)b * c.max_blocks + first + pos / c.block_size];
            dst[u] = ((blk * n_kv_heads + kvh) * c.block_size + pos % c.block_size) * row_bytes + 16 * p;
            const int64_t src = (((int64_t)b * n_tokens + t) * n_kv_heads + kvh) * row_bytes + 16 * p;
            kr[u] = *reinterpret_cast<const uint4 *>(k_in + src);
            vr[u] = *reinterpret_cast<const uint4 *>(v_in + src);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i0 + u * stride < total) {
                *reinterpret_cast<uint4 *>(c.k_blocks + dst[u]) = kr[u];
                *reinterpret_cast<uint4 *>(c.v_blocks + dst[u]) = vr[u];
            }
        }
    }
    __syncthreads();                                           // every thread has read `len` by now
    if (threadIdx.x == 0) {
        if (gridDim.y == 1) {
            c.win_lens[b] = len + n_tokens;
        } else {
            int32_t *arrived = c.plan + 4 * b + 3;
            if (atomicAdd(arrived, 1) == (int)gridDim.y - 1) {
                *arrived = 0;
                c.win_lens[b] = len + n_tokens;
            }
        }
    }
}

// Alg. 1's eviction rule: whole blocks a window of l_cur tokens gives up (0 below l_max).
__device__ __forceinline__ int blocks_to_evict(const CacheDev &c, int l_cur)
{
    const int l_max = c.win_blocks * c.block_size;
    return l_cur >= l_max ? min((l_cur - l_max + c.block_size) / c.block_size, l_cur / c.block_size) : 0;
}

__device__ __forceinline__ void evict_row(CompactShared &s_compact, const CacheDev &c, int64_t row, int32_t n_q_heads,
                                          double beta, int l_cur, bool store_len, int32_t fail_bits)
{
    const int b = (int)(row / n_q_heads), tid = threadIdx.x;
    const int n_ev = blocks_to_evict(c, l_cur);
    const int l_ev = n_ev * c.block_size;
    if (l_ev == 0 && !store_len) return;                       // the same for every workgroup of the sequence
    int p_old = 0;
    if (l_ev > 0) {
        p_old = c.pool_lens[b];
        float *maw = c.a_maw + row * c.win_cap;

        const int start = min(max(c.ctx_cnt[row], 0), c.k_max);
        float unused = 0.f;
        const int total = threshold_compact<false>(s_compact, maw, l_ev, beta / (double)l_cur, c.ctx_idx + row * c.k_max,
                                                   start, c.k_max, p_old, nullptr, unused);
        if (tid == 0) {
            c.ctx_cnt[row] = min(total, c.k_max);
            if (total > c.k_max) atomicOr(c.status, kCacheListFull);
        }
        if (c.a_evicted) {
            float *dst = c.a_evicted + row * (int64_t)c.pool_cap + p_old;
            for (int j = tid; j < l_ev && p_old + j < c.pool_cap; j += kRowBlock) dst[j] = maw[j];
        }
        __syncthreads();                                       // the evicted averages have been read

        // shift down: a step reads [t0 + l_ev, ...) which no earlier step has written (they wrote below t0)
        const int n_stay = l_cur - l_ev;
        for (int t0 = 0; t0 < l_cur; t0 += kRowStep) {
            float x[kPerThread];
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) {
                const int j = t0 + e * kRowBlock + tid;
                x[e] = j < n_stay ? maw[j + l_ev] : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int e = 0; e < kPerThread; ++e) {
                const int j = t0 + e * kRowBlock + tid;
                if (j < l_cur) maw[j] = x[e];                  // entries [n_stay, l_cur) become 0
            }
        }
    }

    // every thread of this workgroup read the sequence's state before a barrier that lies behind it by now
    if (tid == 0) {
        int32_t *arrived = c.plan + 4 * b + 3;
        if (atomicAdd(arrived, 1) == n_q_heads - 1) {
            *arrived = 0;
            if (l_ev > 0) {
                c.plan[4 * b + 0] = l_ev;                      // what was done, for whoever wants to look
                c.plan[4 * b + 1] = l_cur;
                c.plan[4 * b + 2] = p_old;
                c.first_win_block[b] += n_ev;
                c.pool_lens[b] = p_old + l_ev;
            }
            if (l_ev > 0 || store_len) c.win_lens[b] = l_cur - l_ev;
            if (fail_bits) atomicOr(c.status, fail_bits);
        }
    }
}

__global__ __launch_bounds__(kRowBlock) void evict_kernel(CacheDev c, int32_t n_q_heads, double beta)
{
    __shared__ CompactShared s_compact;
    const int l_cur = c.win_lens[blockIdx.x / n_q_heads];
    __syncthreads();
    evict_row(s_compact, c, blockIdx.x, n_q_heads, beta, l_cur, false, 0);
}

// The tail of a decode step over the managed cache as one launch, one workgroup per (sequence, query head) row:
// merge_state over the row's split partials (set p: the window's, set q: the salient list's), the window's attention
// weights A_gpu = e^{s - lse_window} from the scaled scores the split kernels left in a_gpu, Alg. 1's moving average
// (the newest token has no history and takes its first weight), then eviction and sparsification of the row.
// Nothing here needs another row's results, so the three steps need no launch boundary between them; the row's
// scores and averages are requested together with the partials, so the launch costs one round trip to memory.
// With token_pending the step's token was written into the window by the split kernels and its length is still the
// old one: the length this step works with is taken from the same rule (pending_window_len) and stored here.
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(kRowBlock) void decode_tail_kernel(Partials p, Partials q, void *o, float *lse, float *a_gpu,
                                                                CacheDev c, int32_t n_q_heads, float alpha, double beta,
                                                                int32_t token_pending)
{
    static_assert(kFoldBlock == kRowBlock, "one workgroup shape for the fold and the row passes");
    constexpr int PF = 16;                                     // entries per thread requested before the fold
    __shared__ FoldShared<D> s_fold;
    __shared__ CompactShared s_compact;
    const int64_t row = blockIdx.x;
    const int b = (int)(row / n_q_heads), tid = threadIdx.x, cap = c.win_cap;
    float *ar = a_gpu + row * cap;
    float *m = c.a_maw + row * cap;
    float s[PF], h[PF];
#pragma unroll
    for (int e = 0; e < PF; ++e) {
        const int j = tid + e * kRowBlock;
        s[e] = j < cap ? ar[j] : 0.f;                          // beyond the length: not used
        h[e] = j < cap ? m[j] : 0.f;
    }
    int32_t fail_bits = 0;
    const int n = token_pending ? pending_window_len(c.win_lens[b], c.first_win_block[b], 1, cap, c.block_size,
                                                     c.max_blocks, &fail_bits)
                                : c.win_lens[b];
    const int nc = min(max(n, 0), cap);
    const float lse_w = fold_row<D, OUT_BF16, true>(s_fold, p, q, o, lse, nullptr, row);
    // A row that evicts nothing only reports its arrival (the sequence's last row stores the length): that round
    // trip runs beside the weights pass, which reads nothing the arrival changes.
    const bool evicts = blocks_to_evict(c, n) > 0;             // uniform over the sequence's workgroups
    if (!evicts) evict_row(s_compact, c, row, n_q_heads, beta, n, token_pending != 0, fail_bits);

    const float keep = 1.f - alpha;
    auto update = [&](int j, float sj, float hj) {
        const float x = j < nc ? expf(sj - lse_w) : 0.f;
        ar[j] = x;
        if (j < nc) m[j] = j >= nc - 1 ? x : fmaf(alpha, x, keep * hj);
    };
#pragma unroll
    for (int e = 0; e < PF; ++e) {
        const int j = tid + e * kRowBlock;
        if (j < cap) update(j, s[e], h[e]);
    }
    for (int j = PF * kRowBlock + tid; j < cap; j += kRowBlock) update(j, ar[j], m[j]);
    if (evicts) {
        __syncthreads();                                       // the row's averages are written before they are thresholded
        evict_row(s_compact, c, row, n_q_heads, beta, n, token_pending != 0, fail_bits);
    }
}

// The tail of an append turn over the managed cache as one launch, one workgroup per (sequence, query head) row:
// Alg. 1's moving average with the query-averaged A_gpu (the n_new newest entries take their first weight), the
// re-evaluation of Sec. 3.2.2 (the head's salient list is REPLACED by the pool positions with A_cpu > beta / pool
// length, ascending, -1 padded; a list that is too short raises the status bit), then eviction and sparsification of
// the row.  The three steps of a row need nothing from other rows.
__global__ __launch_bounds__(kRowBlock) void append_tail_kernel(CacheDev c, const float *a_gpu, const float *a_cpu,
                                                                int32_t n_q_heads, int32_t n_new, float alpha, double beta)
{
    __shared__ CompactShared s_compact;
    const int64_t row = blockIdx.x;
    const int b = (int)(row / n_q_heads), tid = threadIdx.x;
    const int l_cur = c.win_lens[b];
    // moving average over the window row
    {
        const int n = min(max(l_cur, 0), c.win_cap), first_new = n - min(n_new, n);
        const float keep = 1.f - alpha;
        float *m = c.a_maw + row * c.win_cap;
        const float *a = a_gpu + row * c.win_cap;
        for (int j = tid; j < n; j += kRowBlock) {
            const float x = a[j];
            m[j] = j >= first_new ? x : fmaf(alpha, x, keep * m[j]);
        }
    }
    // re-evaluation over the pool row
    if (c.pool_cap > 0 && a_cpu) {
        const int n_pool = min(max(c.pool_lens[b], 0), c.pool_cap);
        int32_t *idx = c.ctx_idx + row * c.k_max;
        float unused = 0.f;
        const int passing = threshold_compact<false>(s_compact, a_cpu + row * (int64_t)c.pool_cap, n_pool,
                                                     beta / (double)c.pool_lens[b], idx, 0, c.k_max, 0, nullptr, unused);
        const int kept = min(passing, c.k_max);
        if (tid == 0) {
            c.ctx_cnt[row] = kept;
            if (passing > c.k_max) atomicOr(c.status, kCacheListFull);
        }
        for (int j = kept + tid; j < c.k_max; j += kRowBlock) idx[j] = -1;
    }
    __syncthreads();                                           // the averages and the new list are written before the eviction reads them
    evict_row(s_compact, c, row, n_q_heads, beta, l_cur, false, 0);
}

// KV_ctx of Alg. 1 (per head, the salient entries in contiguous storage): the K and V rows of the listed pool
// positions are copied, in list order, behind the rows a head already holds.  One workgroup copies kCtxRows
// listed entries of one (sequence, head): 16 bytes per lane, consecutive lanes on consecutive pieces of a row,
// four loads in flight.  Rows that would land beyond ctx_cap are left out.
constexpr int kCtxRows = 64;

__global__ __launch_bounds__(kRowBlock) void ctx_compact_kernel(CtxCompactArgs a)
{
    __shared__ uint32_t s_row[kCtxRows];

    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * a.sh.n_q_heads + h;
    const int n = a.kv.cap > 0 ? min(max(a.cnt[bh], 0), a.k_max) : 0;
    const int first = a.first_row ? min(max(a.first_row[bh], 0), a.ctx_cap) : 0;
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.cnt_out) a.cnt_out[bh] = (int32_t)min((int64_t)first + n, (int64_t)a.ctx_cap);
    const int t0 = blockIdx.x * kCtxRows;
    if (t0 >= n) return;                         // uniform over the workgroup
    const int nt = min(min(kCtxRows, n - t0), max(a.ctx_cap - first - t0, 0));
    if (nt <= 0) return;
    const RowMap rows = make_row_map<true, kRowBlock>(s_row, a.kv, a.sh.n_kv_heads, b, h / a.sh.group, t0, nt,
                                                      a.idx + bh * a.k_max + t0);
    const int pieces = a.row_bytes / 16, total = nt * pieces;
    const int64_t dst0 = (bh * a.ctx_cap + first + t0) * (int64_t)a.row_bytes;
    constexpr int U = 4;
    for (int base = threadIdx.x; base < total; base += kRowBlock * U) {
        uint4 kr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = min(base + u * kRowBlock, total - 1);
            const int64_t src = (int64_t)rows(i / pieces) * a.row_bytes + 16 * (i % pieces);
            kr[u] = load16_stream(a.kv.k + src);
            vr[u] = load16_stream(a.kv.v + src);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + u * kRowBlock;
            if (i < total) {
                *reinterpret_cast<uint4 *>(a.k_ctx + dst0 + 16 * (int64_t)i) = kr[u];
                *reinterpret_cast<uint4 *>(a.v_ctx + dst0 + 16 * (int64_t)i) = vr[u];
            }
        }
    }
}

}  // namespace

hipError_t launch_ctx_compact(const CtxCompactArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.k_max == 0) return hipSuccess;
    const dim3 grid((a.k_max + kCtxRows - 1) / kCtxRows, a.sh.n_q_heads, a.sh.batch);
    hipLaunchKernelGGL(ctx_compact_kernel, grid, dim3(kRowBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_kv_append(const CacheDev &c, const void *k_in, const void *v_in, const int32_t *active, int32_t batch,
                            int32_t n_kv_heads, int32_t row_bytes, int32_t n_tokens, hipStream_t s)
{
    if (batch == 0 || n_tokens == 0) return hipSuccess;
    // one workgroup per sequence for a token; for N tokens as many as there are rounds of kRowBlock pieces, up to 16
    const int64_t pieces = (int64_t)n_tokens * n_kv_heads * (row_bytes / 16);
    const unsigned parts = (unsigned)std::max<int64_t>(1, std::min<int64_t>(16, pieces / (4 * kRowBlock)));
    hipLaunchKernelGGL(kv_append_kernel, dim3(batch, parts), dim3(kRowBlock), 0, s, c, static_cast<const char *>(k_in),
                       static_cast<const char *>(v_in), active, n_kv_heads, row_bytes, n_tokens);
    return hipGetLastError();
}

hipError_t launch_decode_tail(int head_dim, int64_t n_rows, const Partials &p, const Partials &q, void *o, int o_dtype,
                              float *lse, float *a_gpu, const CacheDev &c, int32_t n_q_heads, float alpha, double beta,
                              int32_t token_pending, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    const dim3 grid((unsigned)n_rows), block(kRowBlock);
#define HGCA_TAIL_CASE(D, BF)                                                                                       \
    if (head_dim == D && o_dtype == (BF ? 1 : 0))                                                                   \
        hipLaunchKernelGGL((decode_tail_kernel<D, BF>), grid, block, 0, s, p, q, o, lse, a_gpu, c, n_q_heads, alpha, beta, \
                           token_pending)
    HGCA_TAIL_CASE(64, false);
    else HGCA_TAIL_CASE(64, true);
    else HGCA_TAIL_CASE(128, false);
    else HGCA_TAIL_CASE(128, true);
    else return hipErrorInvalidValue;
#undef HGCA_TAIL_CASE
    return hipGetLastError();
}

hipError_t launch_append_tail(const CacheDev &c, const float *a_gpu, const float *a_cpu, int32_t batch, int32_t n_q_heads,
                              int32_t n_new, float alpha, double beta, hipStream_t s)
{
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(append_tail_kernel, dim3((unsigned)((int64_t)batch * n_q_heads)), dim3(kRowBlock), 0, s, c, a_gpu, a_cpu,
                       n_q_heads, n_new, alpha, beta);
    return hipGetLastError();
}

hipError_t launch_kv_evict(const CacheDev &c, int32_t batch, int32_t n_q_heads, double beta, hipStream_t s)
{
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(evict_kernel, dim3((unsigned)((int64_t)batch * n_q_heads)), dim3(kRowBlock), 0, s, c, n_q_heads, beta);
    return hipGetLastError();
}

}  // namespace hgca
