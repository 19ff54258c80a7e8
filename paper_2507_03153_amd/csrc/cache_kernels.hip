// KV manager (Alg. 1) for tiers that live in one block pool in HBM: a sequence's KV entries sit in
// fixed-size blocks listed, in arrival order, in one row of a block table; the older pool is the
// first `first_win_block` blocks of the row and the recent window the blocks after them.  Inserting
// a token writes one K and one V row; evicting the oldest window block moves the boundary: no KV row
// is copied.  What does move is the per-entry moving average of attention weights, which is kept
// per window position: the evicted entries' averages are thresholded (Sec. 3.2.2) into the per-head
// lists of salient pool positions and the rest of the row shifts down.
#include "hgca_launch.hpp"
#include "row_map.hpp"
#include "threshold_compact.hpp"

namespace hgca {

namespace {

// One workgroup per sequence: the K and V rows of the n_tokens incoming tokens of every KV head go to the window
// positions len .. len + n_tokens - 1 (slot p % block_size of window block p / block_size); then the length grows.
// A sequence whose window capacity or table row cannot take all of them receives none (status bit).
__global__ __launch_bounds__(kRowBlock) void kv_append_kernel(CacheDev c, const char *k_in, const char *v_in,
                                                              const int32_t *active, int32_t n_kv_heads,
                                                              int32_t row_bytes, int32_t n_tokens)
{
    const int b = blockIdx.x;
    if (active && !active[b]) return;
    const int len = c.win_lens[b];
    const int first = c.first_win_block[b];
    const bool no_room = len + n_tokens > c.win_cap;
    if (len < 0 || no_room || first + (len + n_tokens - 1) / c.block_size >= c.max_blocks) {   // uniform over the workgroup
        if (threadIdx.x == 0) atomicOr(c.status, no_room ? kCacheWindowFull : kCacheContextFull);
        return;
    }
    const int pieces = row_bytes / 16;                         // 16-byte pieces of one row
    const int per_token = n_kv_heads * pieces;
    for (int i = threadIdx.x; i < n_tokens * per_token; i += kRowBlock) {
        const int t = i / per_token, kvh = (i % per_token) / pieces, p = i % pieces;
        const int pos = len + t;
        const int64_t blk = c.block_table[(int64_t)b * c.max_blocks + first + pos / c.block_size];
        const int64_t dst = ((blk * n_kv_heads + kvh) * c.block_size + pos % c.block_size) * row_bytes + 16 * p;
        const int64_t src = (((int64_t)b * n_tokens + t) * n_kv_heads + kvh) * row_bytes + 16 * p;
        *reinterpret_cast<uint4 *>(c.k_blocks + dst) = *reinterpret_cast<const uint4 *>(k_in + src);
        *reinterpret_cast<uint4 *>(c.v_blocks + dst) = *reinterpret_cast<const uint4 *>(v_in + src);
    }
    __syncthreads();                                           // every thread has read `len` by now
    if (threadIdx.x == 0) c.win_lens[b] = len + n_tokens;
}

// Eviction and sparsification of Alg. 1.  One workgroup per (sequence, query head) row.  Every workgroup of a
// sequence takes the same decision from the same state (if l_cur >= l_max: evict the smallest whole number of
// blocks that brings the window below l_max); for a sequence that evicts, the evicted entries whose moving average
// exceeds beta / l_cur join the head's list of salient pool positions (appended in position order), optionally the
// evicted averages are saved at their pool positions, and the row shifts down by l_evict.  The last workgroup of
// the sequence to finish (an arrival counter in plan[4b + 3], left at zero) moves the boundary: by then every
// workgroup of the sequence has read the state it is about to change.
__global__ __launch_bounds__(kRowBlock) void evict_kernel(CacheDev c, int32_t n_q_heads, double beta)
{
    __shared__ CompactShared s_compact;
    const int64_t row = blockIdx.x;
    const int b = (int)(row / n_q_heads), tid = threadIdx.x;
    const int l_cur = c.win_lens[b], l_max = c.win_blocks * c.block_size;
    int n_ev = 0;
    if (l_cur >= l_max) n_ev = min((l_cur - l_max + c.block_size) / c.block_size, l_cur / c.block_size);
    const int l_ev = n_ev * c.block_size;
    if (l_ev == 0) return;                                     // the same for every workgroup of the sequence
    const int p_old = c.pool_lens[b];
    float *maw = c.a_maw + row * c.win_cap;

    const int start = min(max(c.ctx_cnt[row], 0), c.k_max);
    float unused = 0.f;
    const int total = threshold_compact<false>(s_compact, maw, l_ev, beta / (double)l_cur, c.ctx_idx + row * c.k_max, start,
                                        c.k_max, p_old, nullptr, unused);
    if (tid == 0) {
        c.ctx_cnt[row] = min(total, c.k_max);
        if (total > c.k_max) atomicOr(c.status, kCacheListFull);
    }
    if (c.a_evicted) {
        float *dst = c.a_evicted + row * (int64_t)c.pool_cap + p_old;
        for (int j = tid; j < l_ev && p_old + j < c.pool_cap; j += kRowBlock) dst[j] = maw[j];
    }
    __syncthreads();                                           // the evicted averages have been read

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
            if (j < l_cur) maw[j] = x[e];                      // entries [n_stay, l_cur) become 0
        }
    }

    // every thread of this workgroup read the sequence's state before the barriers above
    if (tid == 0) {
        int32_t *arrived = c.plan + 4 * b + 3;
        if (atomicAdd(arrived, 1) == n_q_heads - 1) {
            *arrived = 0;
            c.plan[4 * b + 0] = l_ev;                          // what was done, for whoever wants to look
            c.plan[4 * b + 1] = l_cur;
            c.plan[4 * b + 2] = p_old;
            c.first_win_block[b] += n_ev;
            c.win_lens[b] = l_cur - l_ev;
            c.pool_lens[b] = p_old + l_ev;
        }
    }
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
    hipLaunchKernelGGL(kv_append_kernel, dim3(batch), dim3(kRowBlock), 0, s, c, static_cast<const char *>(k_in),
                       static_cast<const char *>(v_in), active, n_kv_heads, row_bytes, n_tokens);
    return hipGetLastError();
}

hipError_t launch_kv_evict(const CacheDev &c, int32_t batch, int32_t n_q_heads, double beta, hipStream_t s)
{
    if (batch == 0) return hipSuccess;
    hipLaunchKernelGGL(evict_kernel, dim3((unsigned)((int64_t)batch * n_q_heads)), dim3(kRowBlock), 0, s, c, n_q_heads, beta);
    return hipGetLastError();
}

}  // namespace hgca
