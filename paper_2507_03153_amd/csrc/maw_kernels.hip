// The paper's own sparsifier (Alg. 1; Sec. 3.2.2): attention weights of the dense window,
// their moving average, and the per-head threshold rule "keep iff weight > beta / size".
//
// All three are streaming passes over [B*Hq, cap] fp32 rows, a few MB per layer-step: one
// load and at most one store per element, coalesced, no reuse.
#include "hgca_launch.hpp"
#include "threshold_compact.hpp"

namespace hgca {

namespace {

// a[row, j] holds the scaled score s_j on entry; on exit the softmax weight e^{s_j - lse_row}
// (Sec. 2.1, A = softmax(S)) for j < len and 0 beyond.  With maw != nullptr the same pass applies
// Alg. 1's moving-average update to maw[row, j] (see maw_update_kernel).
__global__ __launch_bounds__(kRowBlock) void window_weights_kernel(float *a, const float *lse, const int32_t *seq_lens,
                                                                   int32_t n_q_heads, int32_t cap, float *maw,
                                                                   int32_t n_new, float alpha)
{
    const int64_t row = blockIdx.x;
    const int n = row_len(seq_lens, (int)(row / n_q_heads), cap);
    const int first_new = n - min(n_new, n);
    const float L = lse[row], keep = 1.f - alpha;
    float *p = a + row * cap;
    float *m = maw ? maw + row * cap : nullptr;
    const int j0 = blockIdx.y * kRowStep + threadIdx.x;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int j = j0 + e * kRowBlock;
        if (j < cap) {
            const float x = j < n ? expf(p[j] - L) : 0.f;
            p[j] = x;
            if (m && j < n) m[j] = j >= first_new ? x : fmaf(alpha, x, keep * m[j]);
        }
    }
}

// Alg. 1: A_maw <- (1 - alpha) A_maw + alpha A_gpu on the valid entries of every row; the last
// n_new valid entries have no history and take their first observed weight.
__global__ __launch_bounds__(kRowBlock) void maw_update_kernel(float *maw, const float *a_gpu, const int32_t *seq_lens,
                                                               int32_t n_q_heads, int32_t cap, int32_t n_new,
                                                               float alpha)
{
    const int64_t row = blockIdx.x;
    const int n = row_len(seq_lens, (int)(row / n_q_heads), cap);
    const int first_new = n - min(n_new, n);
    float *m = maw + row * cap;
    const float *a = a_gpu + row * cap;
    const float keep = 1.f - alpha;
    const int j0 = blockIdx.y * kRowStep + threadIdx.x;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int j = j0 + e * kRowBlock;
        if (j < n) {
            const float x = a[j];
            m[j] = j >= first_new ? x : fmaf(alpha, x, keep * m[j]);
        }
    }
}

// One workgroup per (sequence, query head) row: the salient positions in ascending order, -1 padding,
// their count, and optionally the kept weights re-normalised to sum to 1.
__global__ __launch_bounds__(kRowBlock) void threshold_select_kernel(ThresholdArgs a)
{
    __shared__ CompactShared s_compact;
    __shared__ float s_sum[kRowWaves];

    const int64_t row = blockIdx.x;
    const int b = (int)(row / a.n_q_heads);
    const int n = row_len(a.seq_lens, b, a.cap);
    const int size = a.sizes ? a.sizes[b] : a.size_uniform;
    const double thr = a.beta / (double)size;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    int32_t *idx = a.idx + row * a.k_max;
    float *wn = a.w_norm ? a.w_norm + row * a.k_max : nullptr;

    float my_sum = 0.f;
    // with a status word the whole row is examined, so that a list that left entries out is reported
    const int passing = a.status
        ? threshold_compact<false>(s_compact, a.w + row * a.cap, n, thr, idx, 0, a.k_max, 0, wn, my_sum)
        : threshold_compact<true>(s_compact, a.w + row * a.cap, n, thr, idx, 0, a.k_max, 0, wn, my_sum);
    const int kept = min(passing, a.k_max);
    if (a.status && tid == 0 && passing > a.k_max) atomicOr(a.status, a.status_bit);
    for (int j = kept + tid; j < a.k_max; j += kRowBlock) {
        idx[j] = -1;
        if (wn) wn[j] = 0.f;
    }
    if (tid == 0) a.cnt[row] = kept;
    if (!wn) return;

    // re-normalise the kept weights to sum to 1 (fixed reduction order: deterministic)
    my_sum = wave_sum(my_sum);
    if (lane == 0) s_sum[w] = my_sum;
    __syncthreads();                              // also orders the wn stores above before the loads below
    float sum = 0.f;
#pragma unroll
    for (int v = 0; v < kRowWaves; ++v) sum += s_sum[v];
    for (int j = tid; j < kept; j += kRowBlock) wn[j] = wn[j] / sum;
}

}  // namespace

hipError_t launch_window_weights(float *a, const float *lse, const int32_t *seq_lens, int64_t n_rows, int32_t n_q_heads,
                                 int32_t cap, float *maw, int32_t n_new, float alpha, hipStream_t s)
{
    if (n_rows == 0 || cap == 0) return hipSuccess;
    dim3 grid((unsigned)n_rows, (cap + kRowStep - 1) / kRowStep);   // rows in x: no 65 535 limit on them
    hipLaunchKernelGGL(window_weights_kernel, grid, dim3(kRowBlock), 0, s, a, lse, seq_lens, n_q_heads, cap, maw, n_new,
                       alpha);
    return hipGetLastError();
}

hipError_t launch_maw_update(float *maw, const float *a_gpu, const int32_t *seq_lens, int64_t n_rows, int32_t n_q_heads,
                             int32_t cap, int32_t n_new, float alpha, hipStream_t s)
{
    if (n_rows == 0 || cap == 0) return hipSuccess;
    dim3 grid((unsigned)n_rows, (cap + kRowStep - 1) / kRowStep);   // rows in x: no 65 535 limit on them
    hipLaunchKernelGGL(maw_update_kernel, grid, dim3(kRowBlock), 0, s, maw, a_gpu, seq_lens, n_q_heads, cap, n_new,
                       alpha);
    return hipGetLastError();
}

hipError_t launch_threshold_select(const ThresholdArgs &a, int64_t n_rows, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    hipLaunchKernelGGL(threshold_select_kernel, dim3((unsigned)n_rows), dim3(kRowBlock), 0, s, a);
    return hipGetLastError();
}

}  // namespace hgca
