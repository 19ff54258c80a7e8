// Device code of the per-head top-k selection (one workgroup per row of scores); see select_kernels.hip for the
// algorithm.  In a header so that a kernel which runs selection rows beside other work in one launch shares it.
#pragma once

#include "hgca_launch.hpp"

namespace hgca {

namespace {

// 16-byte loads per thread that make up the pre-filter's sample in the 512-thread workgroups (1: 2 048 scores, so
// rows from 4 096 scores on are served; with 2 the ragged batch of 2048 rows is 3 us slower, the others the same)
#ifndef HGCA_SEL_SMALL_SAMPLE_LOADS
#define HGCA_SEL_SMALL_SAMPLE_LOADS 1
#endif
#ifndef HGCA_SEL_BINS
#define HGCA_SEL_BINS 4096
#endif
constexpr int kBins = HGCA_SEL_BINS;
constexpr int kStep = 4 * kWave;                 // scores a wave handles per step
#ifndef HGCA_SEL_SMALL_BLOCK
#define HGCA_SEL_SMALL_BLOCK 512
#endif
constexpr int kLargeBlock = 1024, kSmallBlock = HGCA_SEL_SMALL_BLOCK;   // threads of the workgroup that owns a row
#ifndef HGCA_SEL_CACHE_FLOATS
#define HGCA_SEL_CACHE_FLOATS 33792
#endif
constexpr int kMaxCacheFloats = HGCA_SEL_CACHE_FLOATS;   // 132 KiB of LDS for the padded row

// Larger float <=> larger key; -0.0 and +0.0 map to the same key.
__device__ __forceinline__ uint32_t order_key(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_to_score(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}


struct Binning {
    float lo, inv_w;
    __device__ __forceinline__ float scaled(float s) const { return (s - lo) * inv_w; }
    __device__ __forceinline__ int operator()(float s) const {   // -inf (padding) and NaN land in bin 0
        return max(0, min(kBins - 1, (int)scaled(s)));
    }
};

// The histogram's range is taken over the FINITE scores: an infinite end would make the bin width zero or the scaled
// scores NaN.  Infinite scores (a caller's masked positions, say) then fall into the end bins by clamping.
__device__ __forceinline__ float finite_or(float s, float otherwise) { return fabsf(s) < INFINITY ? s : otherwise; }

// Four consecutive scores starting at position t (a multiple of 4); positions at or beyond n read -inf.
__device__ __forceinline__ float4 load4_padded(const float *sc, bool sc_vec, int t, int n)
{
    if (sc_vec && t + 3 < n) return *reinterpret_cast<const float4 *>(sc + t);
    float4 v = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    if (t < n) v.x = sc[t];
    if (t + 1 < n) v.y = sc[t + 1];
    if (t + 2 < n) v.z = sc[t + 2];
    if (t + 3 < n) v.w = sc[t + 3];
    return v;
}

// Positions below the current lane among the set bits of a lane mask.
__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}


// How a row is held during the passes: re-read from memory every time, cached in LDS as it is (rows of up to
// kMaxCacheFloats scores), or -- for rows up to four times as long -- cached as one byte per score: the upper 7 of
// the 12 bits of its histogram bin, and one flag bit.  A score whose 7 bits differ from those of the threshold bin
// lies above or below the threshold whatever its lower bits are.  The positions that share the threshold's 7 bits
// (about 1 in 128) are listed and read again, all at once, to be counted, collected as candidates of the exact
// ranking, or flagged as kept; the ranking flags the candidates it keeps; so the compaction reads bytes only, and
// the kept scores (they are part of the output) are read again without anything waiting for them.
enum RowMode { kFromMemory = 0, kCachedScores = 1, kCachedBins = 2 };
constexpr int kCoarseShift = 5;                  // histogram bin -> 7 bits of the cached byte
constexpr uint32_t kCoarseMask = 127u, kKeptFlag = 128u;

// Everything that depends on the number of threads of the workgroup that owns a row: 1024 when there are few
// rows (one row per CU: the row is that CU's whole work), 512 when there are many (four workgroups share a CU and
// overlap each other's barriers and memory round trips).
template <int kSelBlock>
struct Sel {
    static constexpr int kSelWaves = kSelBlock / kWave;
    static constexpr int kBinsPerThread = kBins / kSelBlock;
    static constexpr int kMaxCand = kSelBlock;              // one candidate per thread in the exact ranking

    static_assert(kBins >= 2 * kMaxCand, "the candidate lists live in the histogram's space");
    struct SelShared {
        // The histogram is dead once the threshold bin is located; the candidate lists of the exact ranking then
        // take its first 2 * kMaxCand words, and after the ranking the whole array stages the output of the compaction.
        alignas(16) uint32_t hist[kBins];
        __device__ __forceinline__ float *cand_score() { return reinterpret_cast<float *>(hist); }
        __device__ __forceinline__ int32_t *cand_idx() { return reinterpret_cast<int32_t *>(hist + kMaxCand); }
        uint32_t scan_scratch[kSelWaves];
        float wave_min[kSelWaves], wave_max[kSelWaves];
        uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
        uint32_t wave_keq[kSelWaves];                // entries equal to the threshold that are kept, per wave (kCachedBins)
        uint32_t found[2];                           // selected bin / threshold bits, remaining rank
        uint32_t n_cand, n_uncertain;
        __device__ __forceinline__ uint32_t *uncertain() { return hist + 2 * kMaxCand; }
    };

    // Exclusive prefix sum over the workgroup; *total receives the sum of all values.
    static __device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *scratch, uint32_t *total) {
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
    static __device__ __forceinline__ void locate_rank(SelShared &sh, int nb, uint32_t k_rem) {
        constexpr int BPT = kBinsPerThread;          // thread tid owns bins nb-1-BPT*tid .. (descending value)
        const int tid = threadIdx.x;
        uint32_t c[BPT], local = 0;
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            c[i] = (BPT * tid + i < nb) ? sh.hist[nb - 1 - (BPT * tid + i)] : 0u;
            local += c[i];
        }
        uint32_t total;
        uint32_t running = block_exclusive_scan(local, sh.scan_scratch, &total);
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            if (BPT * tid + i < nb && running < k_rem && running + c[i] >= k_rem) {
                sh.found[0] = (uint32_t)(nb - 1 - (BPT * tid + i));
                sh.found[1] = k_rem - running;
            }
            running += c[i];
        }
        __syncthreads();
    }
    // The padded row: wave w owns the positions [w*seg, (w+1)*seg), seg a multiple of kStep; in step i a
    // lane holds the 4 scores at w*seg + kStep*i + 4*lane.  Positions >= n hold -inf.  The row is padded to a
    // whole number of segments (not of workgroups of segments): waves whose segment lies beyond it have no steps.
    // Positions per wave, and the padded length of a row of n scores:
    static __host__ __device__ inline int segment_length(int n) {
        return ((n + kSelWaves - 1) / kSelWaves + kStep - 1) / kStep * kStep;
    }
    static __host__ __device__ inline int padded_length(int n) {
        const int seg = segment_length(n);
        return seg ? (n + seg - 1) / seg * seg : 0;
    }
    // listed positions that share the threshold's 7 bits: whatever the histogram's space holds behind the candidates
    static constexpr int kMaxUncertain = kBins - 2 * kMaxCand;
    static_assert((kBins >> kCoarseShift) <= 128, "a coarse bin and the flag fit a byte");
    static_assert(kBins >= 2 * kMaxCand + kMaxUncertain, "that list lives behind the candidate lists");

    // A thread's view of the padded row: from the LDS copy (CACHED) or from memory.
    template <bool CACHED>
    struct Row {
        const float *sc, *cache;
        bool sc_vec;
        int n, seg;
        __device__ __forceinline__ int padded() const { return (n + seg - 1) / seg * seg; }
        __device__ __forceinline__ int steps() const {             // uniform over a wave
            return (int)(threadIdx.x / kWave) * seg < padded() ? seg / kStep : 0;
        }
        __device__ __forceinline__ int pos(int i) const {
            return (int)(threadIdx.x / kWave) * seg + kStep * i + 4 * (int)(threadIdx.x % kWave);
        }
        __device__ __forceinline__ float4 at(int t) const {
            if (CACHED) return *reinterpret_cast<const float4 *>(cache + t);
            return load4_padded(sc, sc_vec, min(t, (n + 3) / 4 * 4), n);    // clamp: far padding needs no address
        }
    };

    // The usual row, held in REGISTERS: every lane loads its STEPS x 4 scores once, all loads issued before the first
    // is used, and the range, the histogram, the classification against the threshold bin and the ordered
    // compaction all read those registers -- one round trip to memory for the whole row and no copy of it in LDS
    // (a row of 28 672 scores is 7 float4 per lane of a 1024-thread workgroup).  Rows that need more (a threshold
    // bin too crowded to rank its entries one per thread, a tie that the budget cuts, a threshold of -inf) are left
    // untouched: the function then returns false before it has written any output and the caller runs select_row.
    // The caller guarantees segment_length(n) <= STEPS * kStep.
    template <int STEPS>
    static __device__ __forceinline__ bool select_row_in_registers(const SelectArgs &a, SelShared &sh, const float *sc,
                                                                   int32_t *out, int n, int k, int64_t bh)
    {
        const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
        const bool sc_vec = (a.kv.cap & 3) == 0;     // rows start 16-byte aligned
        const int seg = segment_length(n);
        const int padded = (n + seg - 1) / seg * seg;
        const int steps = w * seg < padded ? seg / kStep : 0;        // uniform over a wave
        const int pos0 = w * seg + 4 * lane;                          // position of the lane's first score

        float4 v[STEPS];
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            v[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (i < steps) v[i] = load4_padded(sc, sc_vec, min(pos0 + kStep * i, (n + 3) / 4 * 4), n);
        }
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            const float s[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                mx = fmaxf(mx, s[e]);                                 // padding is -inf: no effect; +inf: see below
                mn = fminf(mn, finite_or(s[e], INFINITY));
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, off, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        }
        if (lane == 0) { sh.wave_min[w] = mn; sh.wave_max[w] = mx; }
        // the padding will be counted into bin 0: start that bin at minus the number of pads
        for (int i = tid; i < kBins; i += kSelBlock) sh.hist[i] = (i == 0) ? (uint32_t)(n - padded) : 0u;
        if (tid == 0) sh.n_cand = 0;
        if (tid < kSelWaves) { sh.wave_gt[tid] = 0; sh.wave_eq[tid] = 0; }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSelWaves; ++i) { mn = fminf(mn, sh.wave_min[i]); mx = fmaxf(mx, sh.wave_max[i]); }
        if (mx == INFINITY) return false;            // a +inf score: the general path takes its range over finite scores (uniform)
        Binning bin;
        bin.lo = mn;
        bin.inv_w = (mx > mn) ? (float)kBins / (mx - mn) : 0.f;

        // histogram, threshold bin
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            if (i < steps) {
                atomicAdd(&sh.hist[bin(v[i].x)], 1u);
                atomicAdd(&sh.hist[bin(v[i].y)], 1u);
                atomicAdd(&sh.hist[bin(v[i].z)], 1u);
                atomicAdd(&sh.hist[bin(v[i].w)], 1u);
            }
        }
        __syncthreads();
        locate_rank(sh, kBins, (uint32_t)k);
        const int tb = (int)sh.found[0];
        const uint32_t k_rem = sh.found[1];          // rank of the k-th entry inside bin tb
        __syncthreads();
        // Bin 0 also holds -inf scores and the topmost bin everything from the maximum on; the two compares below do
        // not see them as inside those bins, so a threshold in an end bin goes to the general path (uniform).
        if (tb == 0 || tb == kBins - 1) return false;

        // entries above the threshold bin are counted, those inside it listed (two compares against the bin's edges;
        // padding fails both)
        const float edge_lo = (float)tb, edge_hi = (float)(tb + 1);
        uint32_t above = 0;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            if (i < steps) {
                const float s[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = bin.scaled(s[e]);
                    const bool over = x >= edge_hi;
                    above += over;
                    if (x >= edge_lo && !over) {
                        const uint32_t slot = atomicAdd(&sh.n_cand, 1u);
                        if (slot < (uint32_t)kMaxCand) { sh.cand_score()[slot] = s[e]; sh.cand_idx()[slot] = pos0 + kStep * i + e; }
                    }
                }
            }
        }
        above = (uint32_t)wave_sum((float)above);    // exact: far below 2^24 per wave
        __syncthreads();
        const uint32_t n_cand = sh.n_cand;
        if (n_cand > (uint32_t)kMaxCand) return false;               // crowded bin (uniform over the workgroup)
        // exact rank of every candidate in (score descending, position ascending) order; up to 64 candidates (the
        // usual case) are ranked by the first wave alone out of its registers, more than that one per thread
        float my_s = 0.f;
        int32_t my_idx = 0;
        if ((uint32_t)tid < n_cand) {
            my_s = sh.cand_score()[tid];
            my_idx = sh.cand_idx()[tid];
        }
        if (n_cand <= (uint32_t)kWave) {
            if (w == 0) {
                uint32_t gt = 0, eq_lower = 0;
                for (uint32_t j = 0; j < n_cand; ++j) {
                    const float sj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_s), j));
                    const int32_t ij = __builtin_amdgcn_readlane(my_idx, j);
                    gt += sj > my_s;
                    eq_lower += (sj == my_s) && (ij < my_idx);
                }
                if ((uint32_t)lane < n_cand && gt + eq_lower == k_rem - 1) {
                    sh.found[0] = __float_as_uint(my_s);
                    sh.found[1] = k_rem - gt;
                }
            }
        } else if ((uint32_t)tid < n_cand) {
            uint32_t gt = 0, eq_lower = 0;
            for (uint32_t j = 0; j < n_cand; ++j) {
                const float sj = sh.cand_score()[j];
                gt += sj > my_s;
                eq_lower += (sj == my_s) && (sh.cand_idx()[j] < my_idx);
            }
            if (gt + eq_lower == k_rem - 1) { sh.found[0] = __float_as_uint(my_s); sh.found[1] = k_rem - gt; }
        }
        __syncthreads();
        const float thr = __uint_as_float(sh.found[0]);
        const uint32_t need_eq = sh.found[1];
        if ((uint32_t)tid < n_cand) {                // per-wave counts of the kept entries: the bin's own ...
            if (my_s > thr) atomicAdd(&sh.wave_gt[my_idx / seg], 1u);
            if (my_s == thr) atomicAdd(&sh.wave_eq[my_idx / seg], 1u);
        }
        if (lane == 0) atomicAdd(&sh.wave_gt[w], above);             // ... and those above it
        __syncthreads();
        uint32_t run = 0, all_eq = 0;
        for (int i = 0; i < kSelWaves; ++i) {
            if (i < w) run += sh.wave_gt[i] + sh.wave_eq[i];
            all_eq += sh.wave_eq[i];
        }
        if (need_eq != all_eq || thr == -INFINITY) return false;     // a tie that the budget cuts: the general path

        // ordered compaction: an entry is kept iff its score is >= T, one lane mask per score gives its place; the
        // lanes of a wave write ascending, mostly adjacent places, so positions and scores go straight to memory
        float *sel = a.sel_scores ? a.sel_scores + bh * a.k_max : nullptr;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            if (i < steps) {
                const float s[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
                bool keep[4];
                uint32_t before = run;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    keep[e] = s[e] >= thr;
                    const unsigned long long m = __ballot(keep[e]);
                    before += lanes_below(m);
                    run += __popcll(m);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (keep[e]) {
                        out[before] = pos0 + kStep * i + e;
                        if (sel) sel[before] = s[e];
                    }
                    before += keep[e];
                }
            }
        }
        return true;
    }

    // Long rows (too long for LDS as fp32) through a PRE-FILTER: a sample of the row (runs of 256
    // scores spread evenly over it) gives an estimate of the score that a little more than the wanted fraction k / n
    // of the row exceeds; one pass over the row then keeps, per wave and in position order, only the scores at or
    // above that estimate (a few per cent of the row) in LDS, and the exact selection -- histogram, threshold bin,
    // exact ranking inside it, ordered compaction -- runs on those few thousand entries.  The row is read once, a
    // score costs one compare, and nothing of the row but the retained entries is written anywhere.  The estimate
    // is only a filter: if fewer than k entries pass it, a wave's list overflows or the threshold bin is crowded,
    // the function returns false before it has written any output and the caller runs select_row.  `lists` is the workgroup's dynamic LDS (list_bytes of it).
    // kSampleLoads 16-byte loads per thread make up the sample (8 for the large workgroups: 32 768 scores).
    static constexpr int kSampleChunk = 256;                     // scores of one run of the sample: what a wave takes with one load
    template <int kSampleLoads>
    static __device__ __forceinline__ bool select_row_prefiltered(const SelectArgs &a, SelShared &sh, float *lists,
                                                                  int list_bytes, const float *sc, int32_t *out, int n,
                                                                  int k, int64_t bh)
    {
        constexpr int kSampleChunks = kSelBlock * kSampleLoads * 4 / kSampleChunk;
        constexpr int kSample = kSampleChunks * kSampleChunk;
        static_assert(kSampleChunks >= 2, "the sample is spread over the row");
        const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
        const bool sc_vec = (a.kv.cap & 3) == 0;     // rows start 16-byte aligned
        const int cap_w = list_bytes / (kSelWaves * 8);              // entries of one wave's list
        // the fraction of the row asked for, raised by six standard deviations of its estimate from the sample
        const float p = (float)k / (float)n;
        const float p_est = p + 6.f * sqrtf(p / (float)kSample) + 8.f / (float)kSample;
        // not worth it (or no room) unless the retained entries are few: uniform over the workgroup
        if (n < 2 * kSample || p_est * (float)n * 1.25f > (float)(cap_w * kSelWaves) || p_est > 0.2f) return false;

        // ---- the sample: range, histogram, the estimate ---------------------------------------------------
        float4 v[kSampleLoads];
#pragma unroll
        for (int u = 0; u < kSampleLoads; ++u) {
            const int j = u * kSelBlock + tid;                       // float4 of the sample
            const int c = j / (kSampleChunk / 4);
            const int start = (int)((int64_t)c * (n - kSampleChunk) / (kSampleChunks - 1)) & ~3;
            v[u] = load4_padded(sc, sc_vec, start + 4 * (j % (kSampleChunk / 4)), n);
        }
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < kSampleLoads; ++u) {
            const float s[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) { mx = fmaxf(mx, finite_or(s[e], -INFINITY)); mn = fminf(mn, finite_or(s[e], INFINITY)); }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, off, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        }
        if (lane == 0) { sh.wave_min[w] = mn; sh.wave_max[w] = mx; }
        for (int i = tid; i < kBins; i += kSelBlock) sh.hist[i] = 0u;
        if (tid == 0) sh.n_cand = 0;
        if (tid < kSelWaves) { sh.wave_gt[tid] = 0; sh.wave_eq[tid] = 0; }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSelWaves; ++i) { mn = fminf(mn, sh.wave_min[i]); mx = fmaxf(mx, sh.wave_max[i]); }
        if (!(mx > mn)) return false;                // a constant sample, or nothing finite in it (uniform)
        Binning bin;
        bin.lo = mn;
        bin.inv_w = (float)kBins / (mx - mn);
#pragma unroll
        for (int u = 0; u < kSampleLoads; ++u) {
            atomicAdd(&sh.hist[bin(v[u].x)], 1u);
            atomicAdd(&sh.hist[bin(v[u].y)], 1u);
            atomicAdd(&sh.hist[bin(v[u].z)], 1u);
            atomicAdd(&sh.hist[bin(v[u].w)], 1u);
        }
        __syncthreads();
        locate_rank(sh, kBins, (uint32_t)min(kSample, (int)ceilf(p_est * (float)kSample)));
        const float floor_score = mn + (float)sh.found[0] * ((mx - mn) / (float)kBins);   // lower edge of that bin
        __syncthreads();

        // ---- the row, once: entries at or above the estimate go to the wave's list, in position order -------
        const int seg = segment_length(n);
        const int padded = (n + seg - 1) / seg * seg;
        const int steps = w * seg < padded ? seg / kStep : 0;        // uniform over a wave
        const int pos0 = w * seg + 4 * lane;
        float *my_score = lists + (size_t)w * 2 * cap_w;             // the wave's list: scores, then positions
        int32_t *my_pos = reinterpret_cast<int32_t *>(my_score + cap_w);
        int held = 0;                                                // entries of the wave's list (uniform over the wave)
        float top = mx;                                              // largest score seen (the sample's or the wave's)
        constexpr int U = 4;                                         // steps whose loads are in flight together
        for (int i0 = 0; i0 < steps; i0 += U) {
            float4 r[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                r[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (i0 + u < steps) r[u] = load4_padded(sc, sc_vec, min(pos0 + kStep * (i0 + u), (n + 3) / 4 * 4), n);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float s[4] = {r[u].x, r[u].y, r[u].z, r[u].w};
                bool keep[4];
                int before = held;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    keep[e] = s[e] >= floor_score;                   // padding (-inf) and NaN fail
                    top = fmaxf(top, s[e]);
                    const unsigned long long m = __ballot(keep[e]);
                    before += (int)lanes_below(m);
                    held += __popcll(m);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (keep[e] && before < cap_w) {
                        my_score[before] = s[e];
                        my_pos[before] = pos0 + kStep * (i0 + u) + e;
                    }
                    before += keep[e];
                }
            }
        }
        return select_from_lists(a, sh, my_score, my_pos, held, cap_w, top, floor_score, seg, out, k, bh);
    }

    // The exact selection among the entries the waves retained (wave w: `held` entries in my_score / my_pos, in position
    // order, all >= floor_score; top: the largest score the wave has seen).  Returns false, before any output is
    // written, if a list overflowed its cap_w entries, fewer than k entries were retained, or the threshold bin is
    // too crowded to rank its entries one per thread.  sh.n_cand, sh.wave_gt and sh.wave_eq must be zero on entry.
    static __device__ __forceinline__ bool select_from_lists(const SelectArgs &a, SelShared &sh, const float *my_score,
                                                             const int32_t *my_pos, int held, int cap_w, float top,
                                                             float floor_score, int seg, int32_t *out, int k, int64_t bh)
    {
        const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
        top = wave_max(top);
        if (lane == 0) { sh.wave_max[w] = top; sh.scan_scratch[w] = (uint32_t)held; }
        for (int i = tid; i < kBins; i += kSelBlock) sh.hist[i] = 0u;
        __syncthreads();
        uint32_t total = 0;
        bool overflow = false;
#pragma unroll
        for (int i = 0; i < kSelWaves; ++i) {
            total += sh.scan_scratch[i];
            overflow |= sh.scan_scratch[i] > (uint32_t)cap_w;
            top = fmaxf(top, sh.wave_max[i]);
        }
        if (overflow || total < (uint32_t)k || !(top > floor_score) || top == INFINITY) return false;   // uniform (+inf: the whole-row path)

        // ---- exact selection among the retained entries (each wave walks its own list) ----------------------
        Binning fine;
        fine.lo = floor_score;
        fine.inv_w = (float)kBins / (top - floor_score);
        for (int j = lane; j < held; j += kWave) atomicAdd(&sh.hist[fine(my_score[j])], 1u);
        __syncthreads();
        locate_rank(sh, kBins, (uint32_t)k);
        const int tb = (int)sh.found[0];
        const uint32_t k_rem = sh.found[1];          // rank of the k-th entry inside bin tb
        __syncthreads();                             // the histogram's space now takes the bin's entries
        uint32_t above = 0;
        for (int j = lane; j < held; j += kWave) {
            const float sj = my_score[j];
            const int b = fine(sj);
            above += b > tb;
            if (b == tb) {
                const uint32_t slot = atomicAdd(&sh.n_cand, 1u);
                if (slot < (uint32_t)kMaxCand) { sh.cand_score()[slot] = sj; sh.cand_idx()[slot] = my_pos[j]; }
            }
        }
        above = (uint32_t)wave_sum((float)above);    // exact: far below 2^24 per wave
        __syncthreads();
        const uint32_t n_cand = sh.n_cand;
        if (n_cand > (uint32_t)kMaxCand) return false;               // crowded bin (uniform over the workgroup)
        float my_s = 0.f;
        int32_t my_idx = 0;
        if ((uint32_t)tid < n_cand) {
            my_s = sh.cand_score()[tid];
            my_idx = sh.cand_idx()[tid];
        }
        if (n_cand <= (uint32_t)kWave) {             // ranked by the first wave alone out of its registers
            if (w == 0) {
                uint32_t gt = 0, eq_lower = 0;
                for (uint32_t j = 0; j < n_cand; ++j) {
                    const float sj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_s), j));
                    const int32_t ij = __builtin_amdgcn_readlane(my_idx, j);
                    gt += sj > my_s;
                    eq_lower += (sj == my_s) && (ij < my_idx);
                }
                if ((uint32_t)lane < n_cand && gt + eq_lower == k_rem - 1) {
                    sh.found[0] = __float_as_uint(my_s);
                    sh.found[1] = k_rem - gt;
                }
            }
        } else if ((uint32_t)tid < n_cand) {         // one entry per thread
            uint32_t gt = 0, eq_lower = 0;
            for (uint32_t j = 0; j < n_cand; ++j) {
                const float sj = sh.cand_score()[j];
                gt += sj > my_s;
                eq_lower += (sj == my_s) && (sh.cand_idx()[j] < my_idx);
            }
            if (gt + eq_lower == k_rem - 1) { sh.found[0] = __float_as_uint(my_s); sh.found[1] = k_rem - gt; }
        }
        __syncthreads();
        const float thr = __uint_as_float(sh.found[0]);
        const uint32_t need_eq = sh.found[1];
        if ((uint32_t)tid < n_cand) {                // per-wave counts of the kept entries: the bin's own ...
            if (my_s > thr) atomicAdd(&sh.wave_gt[my_idx / seg], 1u);
            if (my_s == thr) atomicAdd(&sh.wave_eq[my_idx / seg], 1u);
        }
        if (lane == 0) atomicAdd(&sh.wave_gt[w], above);             // ... and those above it
        __syncthreads();
        uint32_t run_gt = 0, run_eq = 0;             // entries above / equal to T in the lists of the waves before
        for (int i = 0; i < w; ++i) { run_gt += sh.wave_gt[i]; run_eq += sh.wave_eq[i]; }

        // ordered compaction of the lists (they are in position order, wave after wave): kept iff score > T, or
        // score == T and fewer than need_eq equal scores stand before it
        float *sel = a.sel_scores ? a.sel_scores + bh * a.k_max : nullptr;
        for (int j0 = 0; j0 < held; j0 += kWave) {
            const int j = j0 + lane;
            const float sj = j < held ? my_score[j] : -INFINITY;
            const bool gt = sj > thr, eq = sj == thr;
            const unsigned long long m_gt = __ballot(gt), m_eq = __ballot(eq);
            const uint32_t gt_before = run_gt + lanes_below(m_gt), eq_before = run_eq + lanes_below(m_eq);
            if (gt || (eq && eq_before < need_eq)) {
                const uint32_t at = gt_before + min(eq_before, need_eq);
                out[at] = my_pos[j];
                if (sel) sel[at] = sj;
            }
            run_gt += __popcll(m_gt);
            run_eq += __popcll(m_eq);
        }
        return true;
    }

    template <int MODE>
    static __device__ __forceinline__ void select_row(const SelectArgs &a, SelShared &sh, float *cache,
                                                      const float *sc, int32_t *out, int n, int k, int64_t bh)
    {
        constexpr bool CACHED = MODE == kCachedScores, BINS = MODE == kCachedBins;
        uint8_t *cbin = reinterpret_cast<uint8_t *>(cache);         // kCachedBins: one byte per position of the padded row
        const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
        Row<CACHED> row;
        row.sc = sc;
        row.cache = cache;
        row.sc_vec = (a.kv.cap & 3) == 0;            // rows start 16-byte aligned
        row.n = n;
        row.seg = segment_length(n);
        const int padded = row.padded();             // >= n, <= kSelWaves * seg
        const int steps = row.steps();

        // ---- pass 0: range of the row; the padded row goes to LDS ---------------------------------------
        float mn = INFINITY, mx = -INFINITY;
        {
            constexpr int U = 8;                     // 16-byte loads in flight per lane
            const int n4 = padded / 4;
            // kCachedBins: the range is taken from the first kSelBlock * U * 4 scores only.  Any range gives a correct
            // selection (scores beyond it land in the end bins, and a threshold bin that turns out crowded is resolved
            // exactly below); a range that misses part of the row only makes the end bins fuller.
            const int n4_range = BINS ? min(n4, kSelBlock * U) : n4;
            for (int base = 0; base < n4_range; base += kSelBlock * U) {
                float4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    v[u] = load4_padded(sc, row.sc_vec, 4 * min(base + u * kSelBlock + tid, n4 - 1), n);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = base + u * kSelBlock + tid;
                    if (i < n4) {
                        if (CACHED) reinterpret_cast<float4 *>(cache)[i] = v[u];
                        const float s[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            mx = fmaxf(mx, finite_or(s[e], -INFINITY));      // padding is -inf: no effect
                            mn = fminf(mn, finite_or(s[e], INFINITY));
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, off, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        }
        if (lane == 0) { sh.wave_min[w] = mn; sh.wave_max[w] = mx; }
        // the padding will be counted into bin 0: start that bin at minus the number of pads
        for (int i = tid; i < kBins; i += kSelBlock) sh.hist[i] = (i == 0) ? (uint32_t)(n - padded) : 0u;
        if (tid == 0) { sh.n_cand = 0; sh.n_uncertain = 0; }
        if (tid < kSelWaves) { sh.wave_gt[tid] = 0; sh.wave_eq[tid] = 0; sh.wave_keq[tid] = 0; }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSelWaves; ++i) { mn = fminf(mn, sh.wave_min[i]); mx = fmaxf(mx, sh.wave_max[i]); }
        Binning bin;
        bin.lo = mn;
        bin.inv_w = (mx > mn) ? (float)kBins / (mx - mn) : 0.f;

        // ---- pass 1: histogram, threshold bin --------------------------------------------------------------
#pragma unroll 4
        for (int i = 0; i < steps; ++i) {
            const int t = row.pos(i);
            const float4 v = row.at(t);
            const int b0 = bin(v.x), b1 = bin(v.y), b2 = bin(v.z), b3 = bin(v.w);
            atomicAdd(&sh.hist[b0], 1u);
            atomicAdd(&sh.hist[b1], 1u);
            atomicAdd(&sh.hist[b2], 1u);
            atomicAdd(&sh.hist[b3], 1u);
            if (BINS) {
                const uint32_t c0 = b0 >> kCoarseShift, c1 = b1 >> kCoarseShift, c2 = b2 >> kCoarseShift,
                               c3 = b3 >> kCoarseShift;
                *reinterpret_cast<uint32_t *>(cbin + t) = c0 | c1 << 8 | c2 << 16 | c3 << 24;
            }
        }
        __syncthreads();
        locate_rank(sh, kBins, (uint32_t)k);
        const int tb = (int)sh.found[0];
        uint32_t k_rem = sh.found[1];                // rank of the k-th entry inside bin tb
        __syncthreads();

        // ---- pass 2: count the entries above the threshold bin, collect those inside it ---------------------
        // bin(s) > tb and bin(s) == tb are decided on the scaled score itself (two float compares against
        // the bin's edges give the same answer as the truncation and clamps of the histogram pass; the
        // topmost bin has no upper edge; bin 0 has no lower edge: it holds -inf as well, so there every
        // valid position that is not above counts as inside)
        const float edge_lo = (float)tb, edge_hi = (tb == kBins - 1) ? INFINITY : (float)(tb + 1);
        uint32_t above = 0;
        const uint32_t tb7 = (uint32_t)tb >> kCoarseShift;          // kCachedBins: the 7 cached bits of the threshold bin
        auto classify = [&](float sc_e, int pos) {                   // one score against the threshold bin
            bool over, inside;
            if (BINS) {
                // the range of this mode may not cover the row, so scores beyond it sit in the end bins by clamping:
                // the bin itself is compared, not the bin's edges
                const int b = bin(sc_e);
                over = b > tb;
                inside = b == tb && pos < n;
            } else {
                const float x = bin.scaled(sc_e);
                over = tb != kBins - 1 && x >= edge_hi;           // the topmost bin holds +inf as well
                inside = !over && (tb == 0 ? pos < n : x >= edge_lo);    // bin 0 also holds -inf and what lies below the range
            }
            if (inside) {
                const uint32_t slot = atomicAdd(&sh.n_cand, 1u);
                if (slot < (uint32_t)kMaxCand) { sh.cand_score()[slot] = sc_e; sh.cand_idx()[slot] = pos; }
            }
            return over;
        };
        bool use_bytes = BINS;                       // uniform over the workgroup
        if (BINS) {
            for (int i = 0; i < steps; ++i) {
                const int t = row.pos(i);
                const uint32_t bytes = *reinterpret_cast<const uint32_t *>(cbin + t);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t c = (bytes >> (8 * e)) & kCoarseMask;
                    above += c > tb7;
                    if (c == tb7) {
                        const uint32_t slot = atomicAdd(&sh.n_uncertain, 1u);
                        if (slot < (uint32_t)kMaxUncertain) sh.uncertain()[slot] = (uint32_t)(t + e);
                    }
                }
            }
            __syncthreads();
            const uint32_t n_unc = sh.n_uncertain;
            if (n_unc <= (uint32_t)kMaxUncertain) {
                for (uint32_t j = tid; j < n_unc; j += kSelBlock) {  // one round trip to memory for all of them
                    const int pos = (int)sh.uncertain()[j];
                    if (pos >= n) continue;                          // padding
                    if (classify(sc[pos], pos)) {
                        cbin[pos] |= (uint8_t)kKeptFlag;             // above the threshold bin after all: kept
                        atomicAdd(&sh.wave_gt[pos / row.seg], 1u);
                    }
                }
            } else {                                 // too many to list: this row goes on as if it had no cache
                use_bytes = false;
                above = 0;
            }
        }
        if (!use_bytes) {
            for (int i = 0; i < steps; ++i) {
                const int t = row.pos(i);
                const float4 v = row.at(t);
                const float s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) above += classify(s[e], t + e);
            }
        }
        above = (uint32_t)wave_sum((float)above);    // exact: far below 2^24 per wave
        __syncthreads();
        const uint32_t n_cand = sh.n_cand;
        float thr;
        uint32_t need_eq;
        if (n_cand <= (uint32_t)kMaxCand) {
            // exact rank of every candidate in (score descending, position ascending) order; up to 64 candidates
            // (the usual case) are ranked by the first wave alone out of its registers, more than that one per thread
            float my_s = 0.f;
            int32_t my_idx = 0;
            uint32_t eq_lower = 0;                   // candidates with my score at lower positions
            if ((uint32_t)tid < n_cand) {
                my_s = sh.cand_score()[tid];
                my_idx = sh.cand_idx()[tid];
            }
            if (n_cand <= (uint32_t)kWave) {
                if (w == 0) {
                    uint32_t gt = 0;
                    for (uint32_t j = 0; j < n_cand; ++j) {
                        const float sj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_s), j));
                        const int32_t ij = __builtin_amdgcn_readlane(my_idx, j);
                        gt += sj > my_s;
                        eq_lower += (sj == my_s) && (ij < my_idx);
                    }
                    if ((uint32_t)lane < n_cand && gt + eq_lower == k_rem - 1) {
                        sh.found[0] = __float_as_uint(my_s);
                        sh.found[1] = k_rem - gt;
                    }
                }
            } else if ((uint32_t)tid < n_cand) {
                uint32_t gt = 0;
                for (uint32_t j = 0; j < n_cand; ++j) {
                    const float sj = sh.cand_score()[j];
                    gt += sj > my_s;
                    eq_lower += (sj == my_s) && (sh.cand_idx()[j] < my_idx);
                }
                if (gt + eq_lower == k_rem - 1) { sh.found[0] = __float_as_uint(my_s); sh.found[1] = k_rem - gt; }
            }
            __syncthreads();
            thr = __uint_as_float(sh.found[0]);
            need_eq = sh.found[1];
            // per-wave counts of kept-or-tied entries: those above the bin plus the bin's own
            if ((uint32_t)tid < n_cand) {
                if (my_s > thr) atomicAdd(&sh.wave_gt[my_idx / row.seg], 1u);
                if (my_s == thr) atomicAdd(&sh.wave_eq[my_idx / row.seg], 1u);
                if (use_bytes) {                     // the kept candidates are flagged: ties are settled here, by position
                    const bool kept_eq = my_s == thr && eq_lower < need_eq;
                    if (my_s > thr || kept_eq) cbin[my_idx] |= (uint8_t)kKeptFlag;
                    if (kept_eq) atomicAdd(&sh.wave_keq[my_idx / row.seg], 1u);
                }
            }
            if (lane == 0) atomicAdd(&sh.wave_gt[w], above);
            __syncthreads();
        } else {
            // crowded bin: exact radix select (12 + 12 + 8 bits) over the keys of the bin's entries
            use_bytes = false;                       // the bytes cannot tell the entries of one bin apart
            uint32_t prefix = 0, mask = 0;
            const int shifts[3] = {20, 8, 0}, widths[3] = {12, 12, 8};
#pragma unroll
            for (int pass = 0; pass < 3; ++pass) {
                const int shift = shifts[pass], nb = 1 << widths[pass];
                __syncthreads();
                for (int i = tid; i < nb; i += kSelBlock) sh.hist[i] = 0;
                __syncthreads();
                for (int i = 0; i < steps; ++i) {
                    const int t = row.pos(i);
                    const float4 v = row.at(t);
                    const float s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t key = order_key(s[e]);
                        if (t + e < n && bin(s[e]) == tb && (key & mask) == prefix)
                            atomicAdd(&sh.hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
                    }
                }
                __syncthreads();
                locate_rank(sh, nb, k_rem);
                prefix |= sh.found[0] << shift;
                mask |= (uint32_t)(nb - 1) << shift;
                k_rem = sh.found[1];
            }
            thr = key_to_score(prefix);
            need_eq = k_rem;
            // the candidates were not listed: count per wave directly
            uint32_t my_gt = 0, my_eq = 0;
            for (int i = 0; i < steps; ++i) {
                const int t = row.pos(i);
                const float4 v = row.at(t);
                const float s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    my_gt += t + e < n && s[e] > thr;
                    my_eq += t + e < n && s[e] == thr;
                }
            }
            my_gt = (uint32_t)wave_sum((float)my_gt);
            my_eq = (uint32_t)wave_sum((float)my_eq);
            if (lane == 0) { sh.wave_gt[w] = my_gt; sh.wave_eq[w] = my_eq; }
            __syncthreads();
        }

        // ---- pass 3: ordered compaction ----------------------------------------------------------------------
        // The lanes of a wave write ascending, mostly adjacent places, so the kept positions (and scores) go straight
        // to memory.
        int32_t *dst = out;
        float *sel = a.sel_scores ? a.sel_scores + bh * a.k_max : nullptr;
        uint32_t run_gt = 0, run_eq = 0, all_eq = 0; // kept / tied entries before the wave's current step
        for (int i = 0; i < kSelWaves; ++i) {
            if (i < w) { run_gt += sh.wave_gt[i]; run_eq += sh.wave_eq[i]; }
            all_eq += sh.wave_eq[i];
        }
        const bool pad_ties = thr == -INFINITY;      // only then could padding tie with the threshold
        bool sel_deferred = false;                   // the kept scores are fetched after the positions are all known
        if (BINS && use_bytes && !pad_ties) {
            // Every decision is in the bytes by now: kept iff flagged, or in a bin above the threshold's 7 bits.
            // The kept scores are not at hand: fetching each inside this loop would put a round trip to memory into
            // every step, so they are gathered afterwards from the list of kept positions, all at once.
            sel_deferred = sel != nullptr;
            uint32_t run = run_gt;
            for (int i = 0; i < w; ++i) run += sh.wave_keq[i];
            for (int i = 0; i < steps; ++i) {
                const int t = row.pos(i);
                const uint32_t bytes = *reinterpret_cast<const uint32_t *>(cbin + t);
                bool keep[4];
                uint32_t before = run;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t c = (bytes >> (8 * e)) & 255u;
                    keep[e] = (c & kKeptFlag) != 0 || (c & kCoarseMask) > tb7;
                    const unsigned long long m = __ballot(keep[e]);
                    before += lanes_below(m);
                    run += __popcll(m);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (keep[e]) dst[before] = t + e;
                    before += keep[e];
                }
            }
        } else if (need_eq == all_eq && !pad_ties) {
            // Usual case: no tie is cut by the budget, so an entry is kept iff its score is >= T, and one
            // lane mask per score gives its place.
            uint32_t run = run_gt + run_eq;
            for (int i = 0; i < steps; ++i) {
                const int t = row.pos(i);
                const float4 v = row.at(t);
                const float s[4] = {v.x, v.y, v.z, v.w};
                bool keep[4];
                uint32_t before = run;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    keep[e] = s[e] >= thr;
                    const unsigned long long m = __ballot(keep[e]);
                    before += lanes_below(m);
                    run += __popcll(m);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (keep[e]) {
                        dst[before] = t + e;
                        if (sel) sel[before] = s[e];
                    }
                    before += keep[e];
                }
            }
        } else
        for (int i = 0; i < steps; ++i) {
            const int t = row.pos(i);
            const float4 v = row.at(t);
            const float s[4] = {v.x, v.y, v.z, v.w};
            bool gt[4], eq[4];
            uint32_t gt_before = run_gt, eq_before = run_eq;    // entries before this lane's first position
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                gt[e] = s[e] > thr;
                eq[e] = s[e] == thr && !(pad_ties && t + e >= n);
                const unsigned long long m_gt = __ballot(gt[e]), m_eq = __ballot(eq[e]);
                gt_before += lanes_below(m_gt);
                eq_before += lanes_below(m_eq);
                run_gt += __popcll(m_gt);
                run_eq += __popcll(m_eq);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (gt[e] || (eq[e] && eq_before < need_eq)) {
                    const uint32_t at = gt_before + min(eq_before, need_eq);
                    dst[at] = t + e;
                    if (sel) sel[at] = s[e];
                }
                gt_before += gt[e];
                eq_before += eq[e];
            }
        }
        if (sel_deferred) {
            __syncthreads();                         // the positions written above by other threads of the workgroup
            for (int j = tid; j < k; j += kSelBlock) sel[j] = sc[out[j]];
        }
    }
};


// A row of n scores (n >= 1) with budget k (0 < k < n): rows of at most REG_STEPS 256-score steps per wave go through
// the lanes' registers first (REG_STEPS = 0: never); cache_floats / cache_bytes are the padded row lengths up to
// which the workgroup's dynamic LDS (`cache`) holds the row as fp32 / as one byte per score; 0 = that mode is off.
template <int BLOCK, int REG_STEPS>
__device__ __forceinline__ void select_row_any(const SelectArgs &a, typename Sel<BLOCK>::SelShared &sh, float *cache,
                                               const float *sc, int32_t *out, int n, int k, int64_t bh,
                                               int cache_floats, int cache_bytes, int list_bytes)
{
    using S = Sel<BLOCK>;
    if (REG_STEPS > 0 && S::segment_length(n) <= REG_STEPS * kStep) {      // the row fits the lanes' registers
        if (S::template select_row_in_registers<(REG_STEPS > 0 ? REG_STEPS : 1)>(a, sh, sc, out, n, k, bh)) return;
        __syncthreads();                         // the general path starts over on the shared state
    } else if (list_bytes > 0 && S::padded_length(n) > cache_floats) {     // too long for LDS as fp32: pre-filter
        if (S::template select_row_prefiltered<(BLOCK == kLargeBlock ? 8 : HGCA_SEL_SMALL_SAMPLE_LOADS)>(a, sh, cache, list_bytes, sc,
                                                                                                       out, n, k, bh))
            return;
        __syncthreads();                         // the general path starts over on the shared state
    }
    if (S::padded_length(n) <= cache_floats) S::template select_row<kCachedScores>(a, sh, cache, sc, out, n, k, bh);
    else if (S::padded_length(n) <= cache_bytes) S::template select_row<kCachedBins>(a, sh, cache, sc, out, n, k, bh);
    else S::template select_row<kFromMemory>(a, sh, cache, sc, out, n, k, bh);
}

// The whole of one row: budget, count, padding of the list, the trivial cases, then the selection proper.
// `bh` is the row (b * n_q_heads + h); sel_scores rows are addressed with it as well.
template <int BLOCK, int REG_STEPS>
__device__ __forceinline__ void select_one_row(const SelectArgs &a, typename Sel<BLOCK>::SelShared &sh, float *cache,
                                               int64_t bh, int cache_floats, int cache_bytes, int list_bytes)
{
    const int b = (int)(bh / a.sh.n_q_heads);
    const int tid = threadIdx.x;
    const int n = tier_len(a.kv, b);
    int k = a.k_per_seq ? a.k_per_seq[b] : a.k_uniform;
    k = max(0, min(min(k, n), a.k_max));

    const float *sc = a.scores + bh * (int64_t)a.kv.cap;
    int32_t *out = a.idx + bh * (int64_t)a.k_max;

    if (tid == 0) a.cnt[bh] = k;
    for (int j = k + tid; j < a.k_max; j += BLOCK) out[j] = -1;
    if (k == 0) return;
    if (k == n) {                                // everything is kept
        for (int t = tid; t < n; t += BLOCK) {
            out[t] = t;
            if (a.sel_scores) a.sel_scores[bh * (int64_t)a.k_max + t] = sc[t];
        }
        return;
    }
    select_row_any<BLOCK, REG_STEPS>(a, sh, cache, sc, out, n, k, bh, cache_floats, cache_bytes, list_bytes);
}

}  // namespace

}  // namespace hgca
