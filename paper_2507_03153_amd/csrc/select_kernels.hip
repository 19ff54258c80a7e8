// Per-head top-k of the pool scores.  One workgroup per (sequence, query head).
//
// The scores of the row are pulled into LDS once (when they fit), then:
//   1. a 4096-bin histogram over [min, max] of the row locates the bin that holds
//      the k-th largest score (the bin index is a monotone function of the score);
//   2. the few entries of that bin are collected and ranked exactly on their
//      order-preserving 32-bit keys (ties: lower position first), which yields the
//      threshold key T and how many entries equal to T are kept;
//      if the bin is crowded (e.g. many identical scores) an exact 3-pass radix
//      select over the bin's entries does the same job;
//   3. an ordered compaction emits the kept positions in ascending order: every
//      wave owns a contiguous segment and places its entries with ballots and
//      population counts, so the pass needs no barrier per step.
#include "hgca_launch.hpp"

namespace hgca {

namespace {

constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / kWave;
constexpr int kBins = 4096;
constexpr int kMaxCand = 1024;
constexpr int kMaxCacheFloats = 30720;           // 120 KiB of LDS for the row's scores

// Larger float <=> larger key; -0.0 and +0.0 map to the same key.
__device__ __forceinline__ uint32_t order_key(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelShared {
    uint32_t hist[kBins];
    uint32_t cand_key[kMaxCand];
    int32_t cand_idx[kMaxCand];
    uint32_t scan_scratch[kSelWaves];
    float wave_min[kSelWaves], wave_max[kSelWaves];
    uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
    uint32_t found[2];                           // selected bin / key, remaining rank
    uint32_t n_cand;
};

// Exclusive prefix sum over the workgroup; *total receives the sum of all values.
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

// With hist[0..nb) filled: the bin that holds the entry of rank k_rem (1-based, counted from the
// highest bin down) goes to found[0], its rank inside that bin to found[1].
__device__ __forceinline__ void locate_rank(SelShared &sh, int nb, uint32_t k_rem) {
    const int tid = threadIdx.x;
    uint32_t c4[4] = {0, 0, 0, 0}, local = 0;
    if (4 * tid < nb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { c4[i] = sh.hist[nb - 1 - (4 * tid + i)]; local += c4[i]; }
    }
    uint32_t total;
    uint32_t running = block_exclusive_scan(local, sh.scan_scratch, &total);
    if (4 * tid < nb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (running < k_rem && running + c4[i] >= k_rem) {
                sh.found[0] = (uint32_t)(nb - 1 - (4 * tid + i));
                sh.found[1] = k_rem - running;
            }
            running += c4[i];
        }
    }
    __syncthreads();
}

struct Binning {
    float lo, inv_w;
    __device__ __forceinline__ int operator()(float s) const {
        return max(0, min(kBins - 1, (int)((s - lo) * inv_w)));
    }
};

template <bool CACHED>
__device__ __forceinline__ void select_row(const SelectArgs &a, SelShared &sh, float *cache, const float *sc,
                                           int32_t *out, int n, int k)
{
    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const float *data = CACHED ? cache : sc;

    // ---- pass 0: pull the row into LDS, find its range ---------------------------------------
    float mn = INFINITY, mx = -INFINITY;
    for (int t = tid; t < n; t += kSelBlock) {
        const float s = sc[t] + 0.0f;
        if (CACHED) cache[t] = s;
        mn = fminf(mn, s);
        mx = fmaxf(mx, s);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, off, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    }
    if (lane == 0) { sh.wave_min[w] = mn; sh.wave_max[w] = mx; }
    for (int i = tid; i < kBins; i += kSelBlock) sh.hist[i] = 0;
    if (tid == 0) sh.n_cand = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSelWaves; ++i) { mn = fminf(mn, sh.wave_min[i]); mx = fmaxf(mx, sh.wave_max[i]); }
    Binning bin;
    bin.lo = mn;
    bin.inv_w = (mx > mn) ? (float)kBins / (mx - mn) : 0.f;

    // ---- pass 1: histogram, locate the threshold bin ------------------------------------------
    for (int t = tid; t < n; t += kSelBlock) atomicAdd(&sh.hist[bin(data[t])], 1u);
    __syncthreads();
    locate_rank(sh, kBins, (uint32_t)k);
    const int tb = (int)sh.found[0];
    uint32_t k_rem = sh.found[1];                // rank of the k-th entry inside bin tb
    __syncthreads();

    // ---- pass 2: collect the entries of the threshold bin ---------------------------------------
    for (int t = tid; t < n; t += kSelBlock) {
        const float s = data[t];
        if (bin(s) == tb) {
            const uint32_t slot = atomicAdd(&sh.n_cand, 1u);
            if (slot < (uint32_t)kMaxCand) { sh.cand_key[slot] = order_key(s); sh.cand_idx[slot] = t; }
        }
    }
    __syncthreads();
    const uint32_t n_cand = sh.n_cand;
    uint32_t thr, need_eq;
    if (n_cand <= (uint32_t)kMaxCand) {
        // exact rank of every candidate in (key descending, position ascending) order
        if ((uint32_t)tid < n_cand) {
            const uint32_t my_key = sh.cand_key[tid];
            const int32_t my_idx = sh.cand_idx[tid];
            uint32_t gt = 0, eq_lower = 0;
            for (uint32_t j = 0; j < n_cand; ++j) {
                const uint32_t kj = sh.cand_key[j];
                gt += kj > my_key;
                eq_lower += (kj == my_key) && (sh.cand_idx[j] < my_idx);
            }
            if (gt + eq_lower == k_rem - 1) { sh.found[0] = my_key; sh.found[1] = k_rem - gt; }
        }
        __syncthreads();
        thr = sh.found[0];
        need_eq = sh.found[1];
    } else {
        // crowded bin: exact radix select (12 + 12 + 8 bits) over the keys of the bin's entries
        uint32_t prefix = 0, mask = 0;
        const int shifts[3] = {20, 8, 0}, widths[3] = {12, 12, 8};
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = shifts[pass], nb = 1 << widths[pass];
            __syncthreads();
            for (int i = tid; i < nb; i += kSelBlock) sh.hist[i] = 0;
            __syncthreads();
            for (int t = tid; t < n; t += kSelBlock) {
                const float s = data[t];
                const uint32_t key = order_key(s);
                if (bin(s) == tb && (key & mask) == prefix)
                    atomicAdd(&sh.hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
            }
            __syncthreads();
            locate_rank(sh, nb, k_rem);
            prefix |= sh.found[0] << shift;
            mask |= (uint32_t)(nb - 1) << shift;
            k_rem = sh.found[1];
        }
        thr = prefix;
        need_eq = k_rem;
    }

    // ---- pass 3: ordered compaction; wave w owns positions [w*seg, (w+1)*seg) --------------------
    const int seg = ((n + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int beg = min(w * seg, n), end = min(beg + seg, n);
    uint32_t my_gt = 0, my_eq = 0;               // wave-uniform counts of the own segment
    for (int base = beg; base < end; base += kWave) {
        const int t = base + lane;
        uint32_t key = 0;
        if (t < end) key = order_key(data[t]);
        my_gt += __popcll(__ballot(t < end && key > thr));
        my_eq += __popcll(__ballot(t < end && key == thr));
    }
    if (lane == 0) { sh.wave_gt[w] = my_gt; sh.wave_eq[w] = my_eq; }
    __syncthreads();
    uint32_t run_gt = 0, run_eq = 0;
    for (int i = 0; i < w; ++i) { run_gt += sh.wave_gt[i]; run_eq += sh.wave_eq[i]; }
    for (int base = beg; base < end; base += kWave) {
        const int t = base + lane;
        uint32_t key = 0;
        if (t < end) key = order_key(data[t]);
        const bool gt = t < end && key > thr, eq = t < end && key == thr;
        const unsigned long long m_gt = __ballot(gt), m_eq = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        const uint32_t gt_before = run_gt + __popcll(m_gt & below);
        const uint32_t eq_before = run_eq + __popcll(m_eq & below);
        if (gt || (eq && eq_before < need_eq)) out[gt_before + min(eq_before, need_eq)] = t;
        run_gt += __popcll(m_gt);
        run_eq += __popcll(m_eq);
    }
}

__global__ __launch_bounds__(kSelBlock) void select_topk_kernel(SelectArgs a, int cache_floats)
{
    extern __shared__ __attribute__((aligned(16))) float s_cache[];
    __shared__ SelShared sh;

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
    if (k == n) {                                // everything is kept
        for (int t = tid; t < n; t += kSelBlock) out[t] = t;
        return;
    }
    if (n <= cache_floats) select_row<true>(a, sh, s_cache, sc, out, n, k);
    else select_row<false>(a, sh, s_cache, sc, out, n, k);
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t s)
{
    const int64_t rows = (int64_t)a.sh.batch * a.sh.n_q_heads;
    if (rows == 0) return hipSuccess;
    // rows that fit are cached in LDS (dynamic, beyond the 64 KiB default limit)
    const int cache_floats = a.kv.cap <= kMaxCacheFloats ? (a.kv.cap + 3) / 4 * 4 : 0;
    const size_t dyn = (size_t)cache_floats * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(select_topk_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kMaxCacheFloats * (int)sizeof(float));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(select_topk_kernel, dim3((unsigned)rows), dim3(kSelBlock), dyn, s, a, cache_floats);
    return hipGetLastError();
}

}  // namespace hgca
