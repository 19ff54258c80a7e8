// Ordered compaction of the entries of one fp32 row that exceed a threshold (the per-head rule
// "salient iff weight > beta / size"), shared by the kernels that apply it.
#pragma once

#include "hgca_device.hpp"

namespace hgca {

constexpr int kRowBlock = 256;                   // threads of a workgroup that owns one (b, h) row
constexpr int kRowWaves = kRowBlock / kWave;
constexpr int kPerThread = 4;                    // elements a thread handles per step
constexpr int kRowStep = kRowBlock * kPerThread;

__device__ __forceinline__ int32_t row_len(const int32_t *seq_lens, int b, int32_t cap) {
    return seq_lens ? min(max(seq_lens[b], 0), cap) : cap;
}

// Number of lanes below this one whose bit is set in `mask`.
__device__ __forceinline__ int lanes_below_in(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

struct CompactShared {
    int cnt[2][kPerThread][kRowWaves];           // double-buffered: one barrier per step
};

// Called by all kRowBlock threads of a workgroup.  Walks wr[0 .. n) in steps of 1024 entries; sub-round e
// of a step covers entries [e*256, e*256+256) so that loads are coalesced and the output order is the
// position order.  Entry j passes iff (double)wr[j] > thr: the comparison is made in fp64 on the exactly
// widened weight.  The r-th passing entry goes to out[start + r] = j + value_offset (and its weight to
// wn[start + r] if wn != nullptr) as long as start + r < k_max.  Returns start + the number of passing
// entries seen (uniform over the workgroup; may exceed k_max).  With STOP_WHEN_FULL the walk ends once the list
// is full (the return value is then only a lower bound of the count); without it the whole row is examined, so
// that the caller learns whether anything was left out.  my_sum accumulates the weights this thread stored.
template <bool STOP_WHEN_FULL>
__device__ __forceinline__ int threshold_compact(CompactShared &sh, const float *wr, int n, double thr, int32_t *out,
                                                 int start, int k_max, int value_offset, float *wn, float &my_sum)
{
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    int base = start;
    int buf = 0;
    // the loads of a step are issued one step ahead, so a step does not begin with a round trip to memory
    float nx[kPerThread];
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int t = e * kRowBlock + tid;
        nx[e] = t < n ? wr[t] : 0.f;
    }
    for (int t0 = 0; t0 < n && (!STOP_WHEN_FULL || base < k_max); t0 += kRowStep, buf ^= 1) {
        float x[kPerThread];
        bool keep[kPerThread];
        int below[kPerThread];
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) {
            x[e] = nx[e];
            const int tn = t0 + kRowStep + e * kRowBlock + tid;
            nx[e] = tn < n ? wr[tn] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) {
            const int t = t0 + e * kRowBlock + tid;
            keep[e] = t < n && (double)x[e] > thr;
            const uint64_t mask = __ballot(keep[e]);
            below[e] = lanes_below_in(mask);
            if (lane == 0) sh.cnt[buf][e][w] = __popcll(mask);
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) {
            int before = 0, total = 0;
#pragma unroll
            for (int v = 0; v < kRowWaves; ++v) {
                const int c = sh.cnt[buf][e][v];
                before += v < w ? c : 0;
                total += c;
            }
            const int pos = base + before + below[e];
            if (keep[e] && pos < k_max) {
                out[pos] = t0 + e * kRowBlock + tid + value_offset;
                if (wn) wn[pos] = x[e];
                my_sum += x[e];
            }
            base += total;
        }
    }
    return base;
}

}  // namespace hgca
