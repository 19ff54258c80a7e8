// Split-K softmax attention of one decode query per head, and the raw score pass
// used by the selection.  One workgroup = one split of one (sequence, head unit).
//
// Two ways to form the scores of a split:
//   * VALU path (any dtype / head_dim; the gather kernel; fp32): every lane moves
//     16 bytes of a K row, the lanes that share a row reduce their partial dot
//     products with wave shuffles;
//   * MFMA path (bf16, dense over a tier): a wave loads 16-token K tiles with
//     coalesced 16-byte loads, passes them through a padded LDS stage into the
//     A-operand layout of v_mfma_f32_16x16x32_bf16; the B operand holds the query
//     heads of the GQA group (zero-padded to 16 columns), so one K row read serves
//     all heads of the group at no VALU cost.
// After the scores, both paths share the rest: softmax statistics of the split in
// LDS, a V pass with coalesced 16-byte loads and fp32 FMAs, a reduction through
// shuffles and LDS, and one partial (m, l, o) per head and split.
#include "attn_device.hpp"
#include "fold_device.hpp"

namespace hgca {

namespace {

// ---- VALU path -----------------------------------------------------------------------------

template <typename T, int D, int NH, int MODE>
__global__ __launch_bounds__(kBlock) void attn_split_kernel(KernelArgs a)
{
    using SV = SplitValu<T, D, NH, MODE>;
    __shared__ __attribute__((aligned(16))) char s_lds[SV::kLdsBytes];
    SV::run(a, s_lds, blockIdx.x, blockIdx.y, blockIdx.z);
}

#ifndef HGCA_SCORE_PLAIN_STORES_FROM
#define HGCA_SCORE_PLAIN_STORES_FROM 8           // heads per group from which the scores leave with ordinary stores
#endif
#ifndef HGCA_SCORE_WAVES
#define HGCA_SCORE_WAVES 4
#endif
constexpr int kScoreWaves = HGCA_SCORE_WAVES;    // waves per workgroup of the score pass
constexpr int kScoreBlock = kScoreWaves * kWave;

template <int D, int G>
__global__ __launch_bounds__(kScoreBlock) void pool_scores_mfma_kernel(KernelArgs a)
{
    __shared__ uint4 s_stage[kScoreWaves * Stage<D>::kWaveVecs];
    __shared__ __attribute__((aligned(16))) float s_sc[G][kMaxScoreChunk];
    __shared__ uint32_t s_row[kMaxScoreChunk];

    const int chunk_id = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int n = tier_len(a.kv, b);
    const int t0 = chunk_id * a.chunk;
    if (t0 >= n) return;
    const int nt = min(a.chunk, n - t0);
    const int64_t bh0 = (int64_t)b * a.sh.n_q_heads + (int64_t)kvh * G;
    const RowMap rows = make_row_map<false, kScoreBlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0, nt, nullptr);
    mfma_scores<D, G, kMaxScoreChunk, kScoreWaves>(a, s_stage, s_sc, bh0, nt, rows);
    __syncthreads();

    // coalesced streaming stores, 16 bytes per lane where the row alignment allows it
    const int64_t cap = a.kv.cap;
    const bool vec_ok = (cap % 4) == 0;
    const int n4 = (nt + 3) / 4;
    const int n_out = a.group_max ? 1 : G;       // rows written: one per KV head, or one per head
    float *out = a.scores + (a.group_max ? bh0 / G : bh0) * cap + t0;
    for (int i = threadIdx.x; i < n_out * n4; i += kScoreBlock) {
        const int g = i / n4, j = 4 * (i % n4);
        float4 v = *reinterpret_cast<const float4 *>(&s_sc[g][j]);
        if (a.group_max) {
#pragma unroll
            for (int gg = 1; gg < G; ++gg) {
                const float4 u = *reinterpret_cast<const float4 *>(&s_sc[gg][j]);
                v = make_float4(fmaxf(v.x, u.x), fmaxf(v.y, u.y), fmaxf(v.z, u.z), fmaxf(v.w, u.w));
            }
        }
        float *o = out + g * cap + j;
        if (vec_ok && j + 3 < nt) {              // one 16-byte streaming store
            const floatx4 vv = {v.x, v.y, v.z, v.w};
            // Groups of 8 write an eighth of what they read; their scores leave with ordinary stores (measured on
            // the 70B shape: 321 against 332 us per step), smaller groups with non-temporal ones (8B shape: 145
            // against 148 us; MHA: 1040 against 1086 us)
            if (G >= HGCA_SCORE_PLAIN_STORES_FROM) *reinterpret_cast<floatx4 *>(o) = vv;
            else __builtin_nontemporal_store(vv, reinterpret_cast<floatx4 *>(o));
        } else {
            if (j < nt) o[0] = v.x;
            if (j + 1 < nt) o[1] = v.y;
            if (j + 2 < nt) o[2] = v.z;
            if (j + 3 < nt) o[3] = v.w;
        }
    }
}

template <int D, int G>
__global__ __launch_bounds__(kBlock) void dense_attn_mfma_kernel(KernelArgs a)
{
    using DS = DenseSplit<D, G, kBlock>;
    __shared__ __attribute__((aligned(16))) char s_lds[DS::kLdsBytes];
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int n = tier_len(a.kv, b);
    const int t0 = split * a.chunk;
    if (t0 >= n) {
        write_empty_partial<D, G>(a.part, (int64_t)b * a.sh.n_q_heads + (int64_t)kvh * G, split);
        return;
    }
    DS::run(a, s_lds, split, kvh, b, t0, min(a.chunk, n - t0));
}

// ---- combine and merge ------------------------------------------------------------------------------

// One workgroup folds one (b, h) row (fold_device.hpp); lse_p, if given, receives the log-sum-exp of set p alone.
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(kFoldBlock) void combine_kernel(Partials p, Partials q, void *o, float *lse, float *lse_p,
                                                             float *lse_q)
{
    __shared__ FoldShared<D> sh;
    if (lse_p) fold_row<D, OUT_BF16, true>(sh, p, q, o, lse, lse_p, blockIdx.x, lse_q);   // uniform over the launch
    else fold_row<D, OUT_BF16, false>(sh, p, q, o, lse, nullptr, blockIdx.x);
}

// The same fold for MANY rows with few splits each (the append stage: B * N * Hq rows): a workgroup per row would be
// thousands of workgroups of a few KB each.  Here a thread owns four columns of one row and walks the row's splits
// itself, so a workgroup folds kFoldBlock / (D / 4) rows and needs neither LDS nor a barrier.
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(kFoldBlock) void combine_rows_kernel(Partials p, Partials q, void *o, float *lse, float *lse_p,
                                                                  float *lse_q, int64_t n_rows)
{
    constexpr int C4 = D / 4, R = kFoldBlock / C4;
    const int64_t row = (int64_t)blockIdx.x * R + threadIdx.x / C4;
    const int c4 = threadIdx.x % C4;
    if (row >= n_rows) return;
    const int np = p.n_splits, nq = q.n_splits, n = np + nq;
    auto m_of = [&](int s) { return s < np ? p.m[row * np + s] : q.m[row * nq + (s - np)]; };
    auto l_of = [&](int s) { return s < np ? p.l[row * np + s] : q.l[row * nq + (s - np)]; };
    auto o_of = [&](int s) {
        const float *base = s < np ? p.o + (row * np + s) * D : q.o + (row * nq + (s - np)) * D;
        return *reinterpret_cast<const float4 *>(base + 4 * c4);
    };
    float M = -INFINITY;
    for (int s = 0; s < n; ++s) M = fmaxf(M, m_of(s));
    float L = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (M != -INFINITY) {
        for (int s = 0; s < n; ++s) {
            const float wgt = expf(m_of(s) - M);                 // 0 for empty splits (m = -inf)
            const float4 v = o_of(s);
            L = fmaf(l_of(s), wgt, L);
            acc.x = fmaf(v.x, wgt, acc.x); acc.y = fmaf(v.y, wgt, acc.y);
            acc.z = fmaf(v.z, wgt, acc.z); acc.w = fmaf(v.w, wgt, acc.w);
        }
    }
    const float inv = (M != -INFINITY) ? 1.f / L : 0.f;
    const float r[4] = {acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv};
    if (OUT_BF16) {
        uint16_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t u = __float_as_uint(r[e]);
            u += 0x7fffu + ((u >> 16) & 1u);                     // round to nearest even (finite values)
            h[e] = (uint16_t)(u >> 16);
        }
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(o) + row * D + 4 * c4) =
            make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    } else {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(o) + row * D + 4 * c4) = make_float4(r[0], r[1], r[2], r[3]);
    }
    if (c4 == 0 && lse) lse[row] = (M != -INFINITY) ? M + logf(L) : -INFINITY;
    // each set alone, by two other threads of the row
    if ((c4 == 1 && lse_p) || (c4 == 2 && lse_q)) {
        const Partials &t = c4 == 1 ? p : q;
        const int nt = t.n_splits;
        float Mt = -INFINITY, Lt = 0.f;
        for (int s = 0; s < nt; ++s) Mt = fmaxf(Mt, t.m[row * nt + s]);
        if (Mt != -INFINITY)
            for (int s = 0; s < nt; ++s) Lt = fmaf(t.l[row * nt + s], expf(t.m[row * nt + s] - Mt), Lt);
        (c4 == 1 ? lse_p : lse_q)[row] = (Mt != -INFINITY) ? Mt + logf(Lt) : -INFINITY;
    }
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

// ---- launch plumbing ------------------------------------------------------------------------------------

// rows from which the fold takes several rows per workgroup (a thread walks its row's splits itself); measured: 8192
// rows of 8 splits 18 -> 9 us; 2048 rows of ~20 splits 1 us slower than a workgroup per row
#ifndef HGCA_FOLD_MANY_ROWS
#define HGCA_FOLD_MANY_ROWS 4096
#endif

#define HGCA_LAUNCH(kernel, grid, block, stream, ...) \
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__)

template <typename T, int D, int MODE>
hipError_t launch_valu_group(const KernelArgs &ka, int nh, dim3 grid, hipStream_t s)
{
    switch (nh) {
    case 1: HGCA_LAUNCH((attn_split_kernel<T, D, 1, MODE>), grid, dim3(kBlock), s, ka); break;
    case 2: HGCA_LAUNCH((attn_split_kernel<T, D, 2, MODE>), grid, dim3(kBlock), s, ka); break;
    case 4: HGCA_LAUNCH((attn_split_kernel<T, D, 4, MODE>), grid, dim3(kBlock), s, ka); break;
    case 8: HGCA_LAUNCH((attn_split_kernel<T, D, 8, MODE>), grid, dim3(kBlock), s, ka); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D, int MODE>
hipError_t launch_mfma_group(const KernelArgs &ka, int g, dim3 grid, hipStream_t s)
{
#define HGCA_MFMA_CASE(G)                                                                           \
    case G:                                                                                         \
        if (MODE == kScores) HGCA_LAUNCH((pool_scores_mfma_kernel<D, G>), grid, dim3(kScoreBlock), s, ka); \
        else HGCA_LAUNCH((dense_attn_mfma_kernel<D, G>), grid, dim3(kBlock), s, ka);                \
        break;
    switch (g) {
        HGCA_MFMA_CASE(1) HGCA_MFMA_CASE(2) HGCA_MFMA_CASE(4) HGCA_MFMA_CASE(8)
    default: return hipErrorInvalidValue;
    }
#undef HGCA_MFMA_CASE
    return hipGetLastError();
}

// dense / score passes over a tier: bf16 takes the MFMA path, fp32 the VALU path
template <int MODE>
hipError_t launch_tier_pass(int dtype, int head_dim, const KernelArgs &ka, dim3 grid, hipStream_t s)
{
    const int g = ka.sh.group;
    if (dtype == 1 && head_dim == 64) return launch_mfma_group<64, MODE>(ka, g, grid, s);
    if (dtype == 1 && head_dim == 128) return launch_mfma_group<128, MODE>(ka, g, grid, s);
    if (dtype == 0 && head_dim == 64) return launch_valu_group<float, 64, MODE>(ka, g, grid, s);
    if (dtype == 0 && head_dim == 128) return launch_valu_group<float, 128, MODE>(ka, g, grid, s);
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
    ka.sel_scores = a.sel_scores;
    ka.k_max = a.k_max;
    ka.chunk = a.chunk;
    ka.part = a.part;
    ka.scores = a.raw_scores;
    return ka;
}

}  // namespace

hipError_t launch_attn_partial_dense(int dtype, int head_dim, const AttnArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.part.n_splits == 0) return hipSuccess;
    dim3 grid(a.part.n_splits, a.sh.n_kv_heads, a.sh.batch);
    return launch_tier_pass<kDense>(dtype, head_dim, to_kernel_args(a), grid, s);
}

template <typename T, int D>
hipError_t launch_gather_group(const KernelArgs &ka, int nh, dim3 grid, hipStream_t s)
{
    switch (nh) {
    case 1: HGCA_LAUNCH((attn_split_kernel<T, D, 1, kGatherGroup>), grid, dim3(kBlock), s, ka); break;
    case 2: HGCA_LAUNCH((attn_split_kernel<T, D, 2, kGatherGroup>), grid, dim3(kBlock), s, ka); break;
    case 4: HGCA_LAUNCH((attn_split_kernel<T, D, 4, kGatherGroup>), grid, dim3(kBlock), s, ka); break;
    case 8: HGCA_LAUNCH((attn_split_kernel<T, D, 8, kGatherGroup>), grid, dim3(kBlock), s, ka); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attn_partial_gather(int dtype, int head_dim, const AttnArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.part.n_splits == 0) return hipSuccess;
    if (a.grouped) {                             // one list per KV head: a workgroup serves the whole group
        dim3 grid(a.part.n_splits, a.sh.n_kv_heads, a.sh.batch);
        const KernelArgs ka = to_kernel_args(a);
        if (dtype == 0 && head_dim == 64) return launch_gather_group<float, 64>(ka, a.sh.group, grid, s);
        if (dtype == 0 && head_dim == 128) return launch_gather_group<float, 128>(ka, a.sh.group, grid, s);
        if (dtype == 1 && head_dim == 64) return launch_gather_group<bf16_t, 64>(ka, a.sh.group, grid, s);
        if (dtype == 1 && head_dim == 128) return launch_gather_group<bf16_t, 128>(ka, a.sh.group, grid, s);
        return hipErrorInvalidValue;
    }
    dim3 grid(a.part.n_splits, a.sh.n_q_heads, a.sh.batch);
    const KernelArgs ka = to_kernel_args(a);
#define HGCA_GATHER_CASE(T, D)                                                                              \
    if (a.sel_scores) HGCA_LAUNCH((attn_split_kernel<T, D, 1, kGatherScored>), grid, dim3(kBlock), s, ka);  \
    else HGCA_LAUNCH((attn_split_kernel<T, D, 1, kGather>), grid, dim3(kBlock), s, ka)
    if (dtype == 0 && head_dim == 64) { HGCA_GATHER_CASE(float, 64); }
    else if (dtype == 0 && head_dim == 128) { HGCA_GATHER_CASE(float, 128); }
    else if (dtype == 1 && head_dim == 64) { HGCA_GATHER_CASE(bf16_t, 64); }
    else if (dtype == 1 && head_dim == 128) { HGCA_GATHER_CASE(bf16_t, 128); }
    else return hipErrorInvalidValue;
#undef HGCA_GATHER_CASE
    return hipGetLastError();
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
    ka.group_max = a.group_max;
    dim3 grid(a.n_chunks, a.sh.n_kv_heads, a.sh.batch);
    return launch_tier_pass<kScores>(dtype, head_dim, ka, grid, s);
}

hipError_t launch_combine(int head_dim, int64_t n_rows, const Partials &p, float *o, float *lse, hipStream_t s)
{
    Partials none{};
    return launch_combine2(head_dim, n_rows, p, none, o, 0, lse, s);
}

hipError_t launch_combine2(int head_dim, int64_t n_rows, const Partials &p, const Partials &q, void *o, int o_dtype,
                           float *lse, hipStream_t s, float *lse_p, float *lse_q)
{
    if (lse_q && !lse_p) return hipErrorInvalidValue;
    if (n_rows == 0) return hipSuccess;
    if (n_rows >= HGCA_FOLD_MANY_ROWS && p.n_splits + q.n_splits <= 64 && (head_dim == 64 || head_dim == 128)) {
        const int rows_per_wg = kFoldBlock / (head_dim / 4);
        const dim3 grid((unsigned)((n_rows + rows_per_wg - 1) / rows_per_wg)), block(kFoldBlock);
        if (head_dim == 64 && o_dtype == 0) HGCA_LAUNCH((combine_rows_kernel<64, false>), grid, block, s, p, q, o, lse, lse_p, lse_q, n_rows);
        else if (head_dim == 64) HGCA_LAUNCH((combine_rows_kernel<64, true>), grid, block, s, p, q, o, lse, lse_p, lse_q, n_rows);
        else if (o_dtype == 0) HGCA_LAUNCH((combine_rows_kernel<128, false>), grid, block, s, p, q, o, lse, lse_p, lse_q, n_rows);
        else HGCA_LAUNCH((combine_rows_kernel<128, true>), grid, block, s, p, q, o, lse, lse_p, lse_q, n_rows);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)n_rows), block(kFoldBlock);
    if (head_dim == 64 && o_dtype == 0) HGCA_LAUNCH((combine_kernel<64, false>), grid, block, s, p, q, o, lse, lse_p, lse_q);
    else if (head_dim == 64 && o_dtype == 1) HGCA_LAUNCH((combine_kernel<64, true>), grid, block, s, p, q, o, lse, lse_p, lse_q);
    else if (head_dim == 128 && o_dtype == 0) HGCA_LAUNCH((combine_kernel<128, false>), grid, block, s, p, q, o, lse, lse_p, lse_q);
    else if (head_dim == 128 && o_dtype == 1) HGCA_LAUNCH((combine_kernel<128, true>), grid, block, s, p, q, o, lse, lse_p, lse_q);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_merge(int head_dim, int64_t n_rows, const float *o_a, const float *lse_a, const float *o_b,
                        const float *lse_b, void *o_out, int o_dtype, float *lse_out, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    dim3 grid((unsigned)n_rows);
    if (head_dim == 64 && o_dtype == 0)
        HGCA_LAUNCH((merge_kernel<64, false>), grid, dim3(64), s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 64 && o_dtype == 1)
        HGCA_LAUNCH((merge_kernel<64, true>), grid, dim3(64), s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 128 && o_dtype == 0)
        HGCA_LAUNCH((merge_kernel<128, false>), grid, dim3(128), s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else if (head_dim == 128 && o_dtype == 1)
        HGCA_LAUNCH((merge_kernel<128, true>), grid, dim3(128), s, o_a, lse_a, o_b, lse_b, o_out, lse_out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace hgca
