// Group-shared salient lists for grouped-query attention (Sec. 3.3: adjacent heads merged into one sparse
// attention task, with a relaxed per-head sparsification).  The heads of a GQA group read the same K/V
// rows, so one list per KV head lets the sparse part fetch every listed row once per group.
#include "hgca_launch.hpp"

namespace hgca {

namespace {

constexpr int kUBlock = 256;
constexpr int kUWaves = kUBlock / kWave;

// One workgroup per (sequence, KV head): the positions listed by the heads of the group are marked in a bitmap
// in LDS; an ordered walk over the bitmap words then emits the union in ascending order.
__global__ __launch_bounds__(kUBlock) void union_lists_kernel(const int32_t *idx, const int32_t *cnt, int32_t k_max,
                                                              int32_t n_q_heads, int32_t n_kv_heads,
                                                              int32_t n_positions, int32_t *out, int32_t *out_cnt,
                                                              int32_t k_max_out, int32_t *status)
{
    extern __shared__ uint32_t s_bits[];         // one bit per pool position
    __shared__ int s_wave[2][kUWaves];

    const int64_t row = blockIdx.x;
    const int b = (int)(row / n_kv_heads), kvh = (int)(row % n_kv_heads), G = n_q_heads / n_kv_heads;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int words = (n_positions + 31) / 32;
    for (int i = tid; i < words; i += kUBlock) s_bits[i] = 0u;
    __syncthreads();
    for (int g = 0; g < G; ++g) {
        const int64_t h = (int64_t)b * n_q_heads + kvh * G + g;
        const int n = min(max(cnt[h], 0), k_max);
        for (int j = tid; j < n; j += kUBlock) {
            const int p = idx[h * k_max + j];
            if (p >= 0 && p < n_positions) atomicOr(&s_bits[p >> 5], 1u << (p & 31));
        }
    }
    __syncthreads();

    int32_t *dst = out + row * k_max_out;
    int base = 0, buf = 0;                       // entries emitted so far (uniform over the workgroup)
    for (int w0 = 0; w0 < words; w0 += kUBlock, buf ^= 1) {
        uint32_t word = w0 + tid < words ? s_bits[w0 + tid] : 0u;
        const int c = __popc(word);
        int incl = c;                            // inclusive scan over the wave
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int v = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += v;
        }
        if (lane == kWave - 1) s_wave[buf][w] = incl;
        __syncthreads();                         // s_wave is double-buffered: one barrier per step
        int before = 0, total = 0;
#pragma unroll
        for (int v = 0; v < kUWaves; ++v) {
            before += v < w ? s_wave[buf][v] : 0;
            total += s_wave[buf][v];
        }
        int pos = base + before + incl - c;
        while (word) {
            const int bit = __ffs(word) - 1;
            if (pos < k_max_out) dst[pos] = (w0 + tid) * 32 + bit;
            ++pos;
            word &= word - 1;
        }
        base += total;
    }
    for (int j = min(base, k_max_out) + tid; j < k_max_out; j += kUBlock) dst[j] = -1;
    if (tid == 0) {
        out_cnt[row] = min(base, k_max_out);
        if (base > k_max_out && status) atomicOr(status, 1);
    }
}

}  // namespace

hipError_t launch_union_lists(const int32_t *idx, const int32_t *cnt, int32_t k_max, int32_t batch, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t n_positions, int32_t *out, int32_t *out_cnt,
                              int32_t k_max_out, int32_t *status, hipStream_t s)
{
    if (batch == 0) return hipSuccess;
    const size_t lds = (size_t)((n_positions + 31) / 32) * sizeof(uint32_t);
    hipLaunchKernelGGL(union_lists_kernel, dim3((unsigned)((int64_t)batch * n_kv_heads)), dim3(kUBlock), lds, s, idx, cnt,
                       k_max, n_q_heads, n_kv_heads, n_positions, out, out_cnt, k_max_out, status);
    return hipGetLastError();
}

}  // namespace hgca
