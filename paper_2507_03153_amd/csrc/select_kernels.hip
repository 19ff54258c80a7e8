// Per-head top-k of the pool scores: exact radix select on order-preserving
// 32-bit keys (three passes: 12 + 12 + 8 bits, histograms in LDS), then an
// ordered compaction that emits the kept positions in ascending order.
// Equal keys at the threshold are kept lowest position first.
// One workgroup per (sequence, query head).
#include "hgca_launch.hpp"

namespace hgca {

namespace {

constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / kWave;
constexpr int kMaxBins = 4096;

// Larger float <=> larger key; -0.0 and +0.0 map to the same key.
__device__ __forceinline__ uint32_t order_key(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum over the workgroup; *total receives the sum of all values.
// `scratch` holds kSelWaves words; two barriers, scratch reusable afterwards.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *scratch, uint32_t *total) {
    const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) scratch[w] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < kSelWaves; ++i) {
        const uint32_t t = scratch[i];
        if (i < w) before += t;
        all += t;
    }
    __syncthreads();
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(kSelBlock) void select_topk_kernel(SelectArgs a)
{
    __shared__ uint32_t hist[kMaxBins];
    __shared__ uint32_t scan_scratch[kSelWaves];
    __shared__ uint32_t found[2];                // selected bin, remaining rank

    const int64_t bh = blockIdx.x;
    const int b = (int)(bh / a.sh.n_q_heads);
    const int tid = threadIdx.x;
    const int n = tier_len(a.kv, b);
    int k = a.k_per_seq ? a.k_per_seq[b] : a.k_uniform;
    k = max(0, min(min(k, n), a.k_max));

    const float *sc = a.scores + bh * (int64_t)a.kv.cap;
    int32_t *out = a.idx + bh * (int64_t)a.k_max;

    if (tid == 0) a.cnt[bh] = k;
    for (int j = k + tid; j < a.k_max; j += kSelBlock) out[j] = -1;
    if (k == 0) return;

    // ---- radix select: the key of rank k (1-based, descending) -----------------------------
    uint32_t prefix = 0, mask = 0, k_rem = (uint32_t)k;
    const int shifts[3] = {20, 8, 0}, widths[3] = {12, 12, 8};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = shifts[pass], nb = 1 << widths[pass];
        for (int i = tid; i < nb; i += kSelBlock) hist[i] = 0;
        __syncthreads();
        for (int t = tid; t < n; t += kSelBlock) {
            const uint32_t key = order_key(sc[t]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
        }
        __syncthreads();
        // thread `tid` owns the 4 bins nb-1-4*tid .. nb-4-4*tid (descending order of value)
        uint32_t c4[4] = {0, 0, 0, 0}, local = 0;
        if (4 * tid < nb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) { c4[i] = hist[nb - 1 - (4 * tid + i)]; local += c4[i]; }
        }
        uint32_t total;
        uint32_t running = block_exclusive_scan(local, scan_scratch, &total);
        if (4 * tid < nb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (running < k_rem && running + c4[i] >= k_rem) {
                    found[0] = (uint32_t)(nb - 1 - (4 * tid + i));
                    found[1] = k_rem - running;
                }
                running += c4[i];
            }
        }
        __syncthreads();
        prefix |= found[0] << shift;
        mask |= (uint32_t)(nb - 1) << shift;
        k_rem = found[1];
        __syncthreads();
    }
    const uint32_t thr = prefix;                 // key of the k-th largest score
    const uint32_t need_eq = k_rem;              // how many keys equal to thr are kept

    // ---- ordered compaction --------------------------------------------------------------
    uint32_t run_gt = 0, run_eq = 0;
    for (int base = 0; base < n; base += kSelBlock) {
        const int t = base + tid;
        uint32_t gt = 0, eq = 0;
        if (t < n) {
            const uint32_t key = order_key(sc[t]);
            gt = key > thr;
            eq = key == thr;
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan(gt | (eq << 16), scan_scratch, &total);
        const uint32_t gt_before = run_gt + (ex & 0xffffu), eq_before = run_eq + (ex >> 16);
        if (gt || (eq && eq_before < need_eq))
            out[gt_before + min(eq_before, need_eq)] = t;
        run_gt += total & 0xffffu;
        run_eq += total >> 16;
    }
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t s)
{
    const int64_t rows = (int64_t)a.sh.batch * a.sh.n_q_heads;
    if (rows == 0) return hipSuccess;
    hipLaunchKernelGGL(select_topk_kernel, dim3((unsigned)rows), dim3(kSelBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace hgca
