// Split-K softmax attention of one decode query per head (generic VALU path):
// dense over a KV tier (all heads of a GQA group share each K/V row that is
// read), index-gathered per query head, and the raw score pass used by the
// selection.  One workgroup = one split of one (sequence, head unit).
//
// Every lane moves 16 bytes per load; the lanes that share a row reduce their
// partial dot products with wave shuffles; the weights of a split are staged in
// LDS between the K pass and the V pass; the four waves reduce their output
// accumulators through LDS and write one partial (m, l, o) per head and split.
#include "hgca_launch.hpp"

namespace hgca {

namespace {

enum Mode { kDense = 0, kGather = 1, kScores = 2 };

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kUnroll = 4;

struct KernelArgs {
    ShapeDev sh;
    const char *q;
    KvDev kv;
    const int32_t *idx;
    const int32_t *cnt;
    int32_t k_max;
    int32_t chunk;
    Partials part;
    float *scores;
};

template <typename T, int D, int NH, int MODE>
__global__ __launch_bounds__(kBlock) void attn_split_kernel(KernelArgs a)
{
    constexpr int EPL = Elem<T>::kPerLoad;       // elements per lane per load
    constexpr int LPR = D / EPL;                 // lanes per row
    constexpr int RPW = kWave / LPR;             // rows per wave per load
    constexpr int RPI = kWaves * RPW;            // rows per workgroup iteration
    constexpr int ROW_BYTES = D * (int)sizeof(T);

    __shared__ float s_p[NH][kMaxChunk];         // scores of the split, then weights
    __shared__ float s_red[kWaves][NH][D];
    __shared__ float s_m[NH], s_l[NH];

    const int split = blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
    const int Hq = a.sh.n_q_heads, Hkv = a.sh.n_kv_heads;
    const int kvh = (MODE == kGather) ? unit / a.sh.group : unit;
    const int h0 = (MODE == kGather) ? unit : unit * NH;          // first of the NH heads handled
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int r = lane / LPR, c = lane % LPR;

    const int64_t bh0 = (int64_t)b * Hq + h0;
    const int n = (MODE == kGather) ? min(a.cnt[bh0], a.k_max) : tier_len(a.kv, b);
    const int t0 = split * a.chunk;

    if (t0 >= n) {                               // empty split (uniform over the workgroup)
        if (MODE != kScores) {
            for (int i = tid; i < NH * D; i += kBlock) {
                const int g = i / D, col = i % D;
                a.part.o[((bh0 + g) * a.part.n_splits + split) * D + col] = 0.f;
            }
            if (tid < NH) {
                a.part.m[(bh0 + tid) * a.part.n_splits + split] = -INFINITY;
                a.part.l[(bh0 + tid) * a.part.n_splits + split] = 0.f;
            }
        }
        return;
    }
    const int nt = min(a.chunk, n - t0);         // 1 .. chunk tokens in this split
    const int32_t *idx_row = (MODE == kGather) ? a.idx + bh0 * a.k_max + t0 : nullptr;

    float qf[NH][EPL];
#pragma unroll
    for (int g = 0; g < NH; ++g)
        Elem<T>::expand(load16(a.q + ((bh0 + g) * D + c * EPL) * (int64_t)sizeof(T)), qf[g]);

    // ---- K pass: scores of the split into LDS --------------------------------------
    for (int base = 0; base < nt; base += RPI * kUnroll) {
        uint4 kr[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = min(base + u * RPI + w * RPW + r, nt - 1);
            const int32_t tok = (MODE == kGather) ? idx_row[j] : t0 + j;
            kr[u] = load16(a.kv.k + row_offset<ROW_BYTES>(a.kv, Hkv, b, kvh, tok) + c * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * RPI + w * RPW + r;
            float kf[EPL];
            Elem<T>::expand(kr[u], kf);
#pragma unroll
            for (int g = 0; g < NH; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) dot = fmaf(qf[g][e], kf[e], dot);
                dot = group_sum<LPR>(dot);
                if (c == 0 && j < nt) s_p[g][j] = dot * a.sh.sm_scale;
            }
        }
    }
    __syncthreads();

    if (MODE == kScores) {
        for (int i = tid; i < NH * nt; i += kBlock) {
            const int g = i / nt, j = i % nt;
            a.scores[(bh0 + g) * (int64_t)a.kv.cap + t0 + j] = s_p[g][j];
        }
        return;
    }

    // ---- softmax statistics of the split, one wave per head ----------------------------
    for (int g = w; g < NH; g += kWaves) {
        float m = -INFINITY;
        for (int j = lane; j < nt; j += kWave) m = fmaxf(m, s_p[g][j]);
        m = wave_max(m);
        float l = 0.f;
        for (int j = lane; j < nt; j += kWave) {
            const float p = __expf(s_p[g][j] - m);
            s_p[g][j] = p;
            l += p;
        }
        l = wave_sum(l);
        if (lane == 0) { s_m[g] = m; s_l[g] = l; }
    }
    __syncthreads();

    // ---- V pass: o[g][:] = sum_j p[g][j] * v_j ---------------------------------------------
    float acc[NH][EPL];
#pragma unroll
    for (int g = 0; g < NH; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    for (int base = 0; base < nt; base += RPI * kUnroll) {
        uint4 vr[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = min(base + u * RPI + w * RPW + r, nt - 1);
            const int32_t tok = (MODE == kGather) ? idx_row[j] : t0 + j;
            vr[u] = load16(a.kv.v + row_offset<ROW_BYTES>(a.kv, Hkv, b, kvh, tok) + c * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = base + u * RPI + w * RPW + r;
            const bool live = j < nt;
            float vf[EPL];
            Elem<T>::expand(vr[u], vf);
#pragma unroll
            for (int g = 0; g < NH; ++g) {
                const float p = live ? s_p[g][min(j, nt - 1)] : 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
            }
        }
    }

    // rows live in different lane groups of a wave, then in different waves
#pragma unroll
    for (int g = 0; g < NH; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float v = acc[g][e];
#pragma unroll
            for (int off = LPR; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
            if (r == 0) s_red[w][g][c * EPL + e] = v;
        }
    __syncthreads();

    for (int i = tid; i < NH * D; i += kBlock) {
        const int g = i / D, col = i % D;
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) v += s_red[ww][g][col];
        a.part.o[((bh0 + g) * a.part.n_splits + split) * D + col] = v;
    }
    if (tid < NH) {
        a.part.m[(bh0 + tid) * a.part.n_splits + split] = s_m[tid];
        a.part.l[(bh0 + tid) * a.part.n_splits + split] = s_l[tid];
    }
}

// Folds the split partials of one (b, h) row: M = max m_s, L = sum l_s e^{m_s-M},
// O = sum o_s e^{m_s-M} / L, lse = M + ln L.  One thread per output column.
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(Partials p, float *o, float *lse)
{
    const int64_t row = blockIdx.x;
    const int col = threadIdx.x;
    const float *pm = p.m + row * p.n_splits;
    const float *pl = p.l + row * p.n_splits;
    float M = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s) M = fmaxf(M, pm[s]);
    if (M == -INFINITY) {                        // every split empty
        o[row * D + col] = 0.f;
        if (col == 0) lse[row] = -INFINITY;
        return;
    }
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
        const float wgt = expf(pm[s] - M);        // 0 for empty splits (m = -inf)
        L = fmaf(pl[s], wgt, L);
        acc = fmaf(p.o[(row * p.n_splits + s) * D + col], wgt, acc);
    }
    o[row * D + col] = acc / L;
    if (col == 0) lse[row] = M + logf(L);
}

// merge_state on one (b, h) row per workgroup, one thread per column.
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(D) void merge_kernel(const float *o_a, const float *lse_a, const float *o_b,
                                                  const float *lse_b, void *o_out, float *lse_out)
{
    const int64_t row = blockIdx.x;
    const int col = threadIdx.x;
    const float la = lse_a[row], lb = lse_b[row];
    const float m = fmaxf(la, lb);
    float res, lse;
    if (m == -INFINITY) {
        res = 0.f;
        lse = -INFINITY;
    } else {
        const float ea = expf(la - m), eb = expf(lb - m), z = ea + eb;
        const float va = o_a[row * D + col], vb = o_b[row * D + col];
        res = (ea * va + eb * vb) / z;
        lse = m + logf(z);
    }
    __syncthreads();                             // all reads of the row precede aliased writes
    if (OUT_BF16) {
        uint32_t u = __float_as_uint(res);
        u += 0x7fffu + ((u >> 16) & 1u);         // round to nearest even (finite values)
        reinterpret_cast<uint16_t *>(o_out)[row * D + col] = (uint16_t)(u >> 16);
    } else {
        reinterpret_cast<float *>(o_out)[row * D + col] = res;
    }
    if (lse_out && col == 0) lse_out[row] = lse;
}

template <typename T, int D, int MODE>
hipError_t launch_split(const KernelArgs &ka, int nh, dim3 grid, hipStream_t s)
{
    switch (nh) {
    case 1: hipLaunchKernelGGL((attn_split_kernel<T, D, 1, MODE>), grid, dim3(kBlock), 0, s, ka); break;
    case 2: hipLaunchKernelGGL((attn_split_kernel<T, D, 2, MODE>), grid, dim3(kBlock), 0, s, ka); break;
    case 4: hipLaunchKernelGGL((attn_split_kernel<T, D, 4, MODE>), grid, dim3(kBlock), 0, s, ka); break;
    case 8: hipLaunchKernelGGL((attn_split_kernel<T, D, 8, MODE>), grid, dim3(kBlock), 0, s, ka); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int MODE>
hipError_t dispatch_split(int dtype, int head_dim, const KernelArgs &ka, int nh, dim3 grid, hipStream_t s)
{
    if (dtype == 0 && head_dim == 64) return launch_split<float, 64, MODE>(ka, nh, grid, s);
    if (dtype == 0 && head_dim == 128) return launch_split<float, 128, MODE>(ka, nh, grid, s);
    if (dtype == 1 && head_dim == 64) return launch_split<bf16_t, 64, MODE>(ka, nh, grid, s);
    if (dtype == 1 && head_dim == 128) return launch_split<bf16_t, 128, MODE>(ka, nh, grid, s);
    return hipErrorInvalidValue;
}

KernelArgs to_kernel_args(const AttnArgs &a)
{
    KernelArgs ka{};
    ka.sh = a.sh;
    ka.q = static_cast<const char *>(a.q);
    ka.kv = a.kv;
    ka.idx = a.idx;
    ka.cnt = a.cnt;
    ka.k_max = a.k_max;
    ka.chunk = a.chunk;
    ka.part = a.part;
    ka.scores = nullptr;
    return ka;
}

}  // namespace

hipError_t launch_attn_partial_dense(int dtype, int head_dim, const AttnArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.part.n_splits == 0) return hipSuccess;
    dim3 grid(a.part.n_splits, a.sh.n_kv_heads, a.sh.batch);
    return dispatch_split<kDense>(dtype, head_dim, to_kernel_args(a), a.sh.group, grid, s);
}

hipError_t launch_attn_partial_gather(int dtype, int head_dim, const AttnArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.part.n_splits == 0) return hipSuccess;
    dim3 grid(a.part.n_splits, a.sh.n_q_heads, a.sh.batch);
    return dispatch_split<kGather>(dtype, head_dim, to_kernel_args(a), 1, grid, s);
}

hipError_t launch_scores(int dtype, int head_dim, const ScoreArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.n_chunks == 0) return hipSuccess;
    KernelArgs ka{};
    ka.sh = a.sh;
    ka.q = static_cast<const char *>(a.q);
    ka.kv = a.kv;
    ka.chunk = a.chunk;
    ka.scores = a.scores;
    dim3 grid(a.n_chunks, a.sh.n_kv_heads, a.sh.batch);
    return dispatch_split<kScores>(dtype, head_dim, ka, a.sh.group, grid, s);
}

hipError_t launch_combine(int head_dim, int64_t n_rows, const Partials &p, float *o, float *lse, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    if (head_dim == 64)
        hipLaunchKernelGGL((combine_kernel<64>), dim3((unsigned)n_rows), dim3(64), 0, s, p, o, lse);
    else if (head_dim == 128)
        hipLaunchKernelGGL((combine_kernel<128>), dim3((unsigned)n_rows), dim3(128), 0, s, p, o, lse);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_merge(int head_dim, int64_t n_rows, const float *o_a, const float *lse_a, const float *o_b,
                        const float *lse_b, void *o_out, int o_dtype, float *lse_out, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    dim3 grid((unsigned)n_rows);
    if (head_dim == 64 && o_dtype == 0)
        hipLaunchKernelGGL((merge_kernel<64, false>), grid, dim3(64), 0, s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 64 && o_dtype == 1)
        hipLaunchKernelGGL((merge_kernel<64, true>), grid, dim3(64), 0, s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 128 && o_dtype == 0)
        hipLaunchKernelGGL((merge_kernel<128, false>), grid, dim3(128), 0, s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 128 && o_dtype == 1)
        hipLaunchKernelGGL((merge_kernel<128, true>), grid, dim3(128), 0, s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace hgca
