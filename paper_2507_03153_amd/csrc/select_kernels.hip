// Per-head top-k of the pool scores.  One workgroup per (sequence, query head).
//
//   0. the row is pulled into LDS once (when it fits), padded with -inf to a whole
//      number of 256-score steps per wave, and its [min, max] is found;
//   1. a 4096-bin histogram over [min, max] locates the bin that holds the k-th
//      largest score (the bin index is a monotone function of the score);
//   2. entries above that bin are counted per wave; the few entries inside it are
//      collected and ranked exactly (score descending, position ascending), which
//      yields the threshold score T and how many entries equal to T are kept; if
//      the bin is crowded (e.g. many identical scores) an exact 3-pass radix select
//      over order-preserving 32-bit keys of the bin's entries does the same job;
//   3. an ordered compaction emits the kept positions in ascending order: every
//      wave owns a contiguous segment and places its entries with the lane masks
//      of the comparisons, so the pass needs no barrier per step; positions are
//      staged in LDS and leave with coalesced stores.
//
// Rows that do not sit in LDS as fp32 (beyond 33 792 scores for the large workgroups, beyond 4 096 for the small
// ones) first try a sampled pre-filter (select_row_prefiltered): an estimate of the threshold from a sample of the
// row (32 768 scores, 2 048 in the small workgroups: runs of 256 spread evenly over the row), one pass over the row
// that retains the few per cent at or above it in LDS, and the steps above on the retained entries only.  It gives
// the same result or gives up (then the steps above run on the whole row, held as one byte per score or re-read
// from memory).  Measured: 256 rows of 122 880 scores, k = 4096: 63 -> 38 us; 1280 rows of 14 336, k = 1024:
// 48 -> 35 us; 2048 rows of 14 336, k = 1433: 68 -> 51 us; 512 rows of 50 000, k = 2500: 53 -> 32 us.
//
// A row is one CU's work; with a handful of VALU operations per score and pass the
// kernel is bound by that CU's instruction issue, so the passes are kept lean
// (no validity tests thanks to the padding, float compares instead of integer
// keys, 4 scores per lane and step).  The workgroup has 1024 threads when there is at
// most one row per CU and 512 when there are more (the rule and the measurements behind it
// stand at the launch).
#include "select_device.hpp"

#include <algorithm>
#include <atomic>

namespace hgca {

namespace {

// 256-score steps per wave up to which a row is held in the lanes' registers (0: never)
#ifndef HGCA_SEL_REG_STEPS_LARGE
#define HGCA_SEL_REG_STEPS_LARGE 8
#endif
#ifndef HGCA_SEL_REG_STEPS_SMALL
#define HGCA_SEL_REG_STEPS_SMALL 0
#endif

// 1: rows too long for LDS as fp32 go through the sampled pre-filter first (large workgroups only)
#ifndef HGCA_SEL_PREFILTER
#define HGCA_SEL_PREFILTER 1
#endif
#ifndef HGCA_SEL_PREFILTER_SMALL
#define HGCA_SEL_PREFILTER_SMALL 1
#endif

// One workgroup per (sequence, query head) row.  The small workgroups are held to 64 registers per lane so that
// four of them fit a compute unit.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK, BLOCK == kLargeBlock ? 1 : 8) void select_topk_kernel(SelectArgs a, int cache_floats,
                                                                                        int cache_bytes, int list_bytes)
{
    using S = Sel<BLOCK>;
    extern __shared__ __attribute__((aligned(16))) float s_cache[];
    __shared__ typename S::SelShared sh;
    select_one_row<BLOCK, (BLOCK == kLargeBlock ? HGCA_SEL_REG_STEPS_LARGE : HGCA_SEL_REG_STEPS_SMALL)>(
        a, sh, s_cache, blockIdx.x, cache_floats, cache_bytes, list_bytes);
}

// The launch uses the small workgroups when there are more rows than compute units (256 on the MI355X) and two
// small workgroups with a row's bytes fit one unit's LDS: then several workgroups share a unit and one's memory round
// trips and barriers hide behind another's work, which a single large workgroup cannot do for itself.  With one row
// per unit or fewer, or with rows so long that a unit holds one workgroup either way, the large workgroup's 16 waves
// finish a row sooner.  (Measured on rows of 14336 scores: 1280 rows 59 -> 48 us, 2048 rows 94 -> 68 us; 2048 rows
// of 1024 scores 52 -> 22 us; 512 rows of 65536 scores 76 -> 91 us, hence the limit.)
constexpr int kComputeUnits = 256;
constexpr int kSmallMaxPadded = 60 * 1024;       // bytes of a row cached by a small workgroup
constexpr int kSmallCacheFloats = 4096;          // small workgroups keep short rows as fp32 (16 KiB), longer ones as bytes

template <int BLOCK>
hipError_t launch_select_block(const SelectArgs &a, int64_t rows, int max_cache_floats, hipStream_t s)
{
    using S = Sel<BLOCK>;
    // rows whose padded length fits are cached in LDS (dynamic, beyond the 64 KiB default limit)
    // (the padded length grows with n in steps, so the capacity's padded length covers every row)
    const int padded = S::padded_length(a.kv.cap);
    const int cache_floats = padded <= max_cache_floats ? padded : 0;
    // longer rows, up to four times the large cache: one byte per score
    const int cache_bytes = cache_floats == 0 && padded <= 4 * kMaxCacheFloats ? padded : 0;
    // once per device: lift the dynamic LDS limit of the kernel (the attribute belongs to a device's copy of it)
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> limit_lifted[kMaxDevices];          // zero-initialised
    int dev = 0;
    hipError_t rc = hipGetDevice(&dev);
    if (rc != hipSuccess) return rc;
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (!tracked || !limit_lifted[dev].load(std::memory_order_acquire)) {
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(select_topk_kernel<BLOCK>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, kMaxCacheFloats * (int)sizeof(float));
        if (rc != hipSuccess) return rc;
        if (tracked) limit_lifted[dev].store(true, std::memory_order_release);
    }
    // rows that do not fit as fp32 try the pre-filter first when the workgroup is alone on its unit: its lists take
    // the whole dynamic allocation (the byte cache of the general path, if that runs after all, uses the same memory)
    // (the small workgroups, when asked to, keep their lists in the allocation of their byte cache)
    const int list_bytes = !HGCA_SEL_PREFILTER || cache_floats != 0 ? 0
                           : BLOCK == kLargeBlock ? kMaxCacheFloats * (int)sizeof(float)
                           : HGCA_SEL_PREFILTER_SMALL && cache_bytes ? std::min(kSmallMaxPadded, 2 * cache_bytes) : 0;
    const size_t lds = cache_floats ? (size_t)cache_floats * sizeof(float)
                                    : std::max((size_t)cache_bytes, (size_t)list_bytes);
    hipLaunchKernelGGL(select_topk_kernel<BLOCK>, dim3((unsigned)rows), dim3(BLOCK), lds, s, a, cache_floats,
                       cache_bytes, list_bytes);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t s)
{
    const int64_t rows = (int64_t)a.sh.batch * a.sh.n_q_heads;
    if (rows == 0) return hipSuccess;
    if (rows > kComputeUnits && Sel<kSmallBlock>::padded_length(a.kv.cap) <= kSmallMaxPadded)
        return launch_select_block<kSmallBlock>(a, rows, kSmallCacheFloats, s);
    return launch_select_block<kLargeBlock>(a, rows, kMaxCacheFloats, s);
}

}  // namespace hgca
