// Append stage: N queries per sequence attend to one KV tier (Sec. 2.1: S = Q K^T, A = softmax(S),
// O = A V with Q in R^{h x N x d}; Alg. 2, append branch).  bf16 inputs, both contractions on
// v_mfma_f32_16x16x32_bf16.
//
// Work unit: one workgroup = one split of the tokens of one (sequence, KV head) and up to 128 query
// rows (a row = one query x one head of the GQA group, query-major).  The four waves own disjoint
// 16-row tiles (wave w: tiles w and w+4), so nothing is reduced across waves; all 256 threads stage
// the K and V rows of a 32-token step into LDS with coalesced 16-byte loads (next step's loads in
// flight during the current step's arithmetic, double-buffered stage, one barrier per step).
//
// Orientation (per 16-row tile, per step):
//   S^T[token, row]  = K[token, :] . Q[row, :]        A = K tile (LDS, padded rows), B = Q (registers)
//   O^T[dcol, row]  += V^T[dcol, token] . P^T[token, row]   A = V^T (LDS, read 2 bytes at a time), B = P
// In both results a lane's column is the query row lane%16, so the running maximum, the running sum
// and the rescaling factor of a row live in the lanes that hold its scores AND its output columns:
// the online softmax needs two shuffles per row statistic and no LDS.  The probabilities go from
// the score registers straight into the B operand of the second contraction (the contraction index
// is matched by reading V^T in the same token order); they are rounded to bf16 there, optionally as
// a high and a low part (two MFMAs) to keep fp32-level accuracy.
#include "hgca_launch.hpp"
#include "row_map.hpp"

namespace hgca {

namespace {

constexpr int kABlock = 256;
constexpr int kAWaves = kABlock / kWave;
constexpr int kStepTokens = 32;
constexpr int kRowsPerBlock = 128;               // query rows per workgroup = 8 tiles of 16
constexpr int kTilesPerWave = kRowsPerBlock / 16 / kAWaves;
constexpr int kSub = kMaxChunk;                  // tokens per refill of the row table

template <int D> struct AStage {
    static constexpr int kPieces = D / 8;                        // 16-byte pieces per row
    static constexpr int kKStride = kPieces + 1;                 // K row stride in uint4 (conflict-free b128 reads)
    static constexpr int kVStride = D * 2 + 8;                   // V row stride in bytes (conflict-free 2-byte reads)
    static constexpr int kLoads = kStepTokens * kPieces / kABlock;   // 16-byte loads per thread, step and tensor
};

__device__ __forceinline__ uint32_t bf16_rne(float x) {          // finite x
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Token of the step that contraction index 8*g + i stands for in lane group g: the lane's own score
// registers hold tokens 4g..4g+3 of the step's first 16-token tile and of its second one.
__device__ __forceinline__ int step_token(int g, int i) { return i < 4 ? 4 * g + i : 16 + 4 * g + (i - 4); }

// Row bookkeeping of one 16-row tile for this lane (column n = lane % 16).
struct RowInfo {
    bool valid;
    int query;
    int64_t out_row;                             // (b * N + query) * Hq + head
};

template <int G>
__device__ __forceinline__ RowInfo row_info(const AppendArgs &a, int b, int kvh, int r) {
    RowInfo ri;
    ri.valid = r < a.n_q * G;
    ri.query = ri.valid ? r / G : 0;
    ri.out_row = ((int64_t)b * a.n_q + ri.query) * a.sh.n_q_heads + kvh * G + (ri.valid ? r % G : 0);
    return ri;
}

template <int D>
__device__ __forceinline__ void load_q_tile(const AppendArgs &a, const RowInfo &ri, int g, bf16x8 (&qop)[D / 32]) {
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        uint4 r = make_uint4(0u, 0u, 0u, 0u);
        if (ri.valid) r = load16(static_cast<const char *>(a.q) + (ri.out_row * D + 32 * kk + 8 * g) * 2);
        qop[kk] = __builtin_bit_cast(bf16x8, r);
    }
}

// Stages the K (and V) rows of 32-token steps: global -> registers -> LDS, one step ahead.
template <int D, bool WITH_V>
struct StepLoader {
    using S = AStage<D>;
    static constexpr size_t ROW_BYTES = D * 2;
    uint4 kr[S::kLoads], vr[S::kLoads];

    __device__ __forceinline__ void fetch(const KvDev &kv, const RowMap &rows, int step, int nsub) {
#pragma unroll
        for (int u = 0; u < S::kLoads; ++u) {
            const int p = threadIdx.x + kABlock * u, trow = p / S::kPieces, piece = p % S::kPieces;
            const int j = min(step * kStepTokens + trow, nsub - 1);
            const size_t off = rows(j) * ROW_BYTES + 16 * piece;
            kr[u] = load16_stream(kv.k + off);
            if (WITH_V) vr[u] = load16_stream(kv.v + off);
        }
    }
    __device__ __forceinline__ void park(uint4 *s_k, char *s_v) const {
#pragma unroll
        for (int u = 0; u < S::kLoads; ++u) {
            const int p = threadIdx.x + kABlock * u, trow = p / S::kPieces, piece = p % S::kPieces;
            s_k[trow * S::kKStride + piece] = kr[u];
            if (WITH_V) {
                char *dst = s_v + trow * S::kVStride + 16 * piece;
                *reinterpret_cast<uint2 *>(dst) = make_uint2(vr[u].x, vr[u].y);
                *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(vr[u].z, vr[u].w);
            }
        }
    }
};

// Scaled, masked scores of one 16-row tile for the step's 32 tokens: sv[4*tt + r] belongs to step token
// 16*tt + 4*g + r and query row lane % 16.  Tokens at or beyond `limit` (counted from the step's first
// token) read -inf.
template <int D>
__device__ __forceinline__ void tile_scores(const uint4 *s_k, const bf16x8 (&qop)[D / 32], float scale, int limit,
                                            float (&sv)[8])
{
    using S = AStage<D>;
    const int lane = threadIdx.x % kWave, n = lane % 16, g = lane / 16;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            const uint4 ka = s_k[(tt * 16 + n) * S::kKStride + 4 * kk + g];
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qop[kk], c, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sv[4 * tt + r] = (16 * tt + 4 * g + r < limit) ? c[r] * scale : -INFINITY;
    }
}

template <int D, int G, bool SPLIT_P>
__global__ __launch_bounds__(kABlock) void append_attn_kernel(AppendArgs a)
{
    using S = AStage<D>;
    constexpr int DT = D / 16;
    __shared__ uint4 s_k[2][kStepTokens * S::kKStride];
    __shared__ __attribute__((aligned(16))) char s_v[2][kStepTokens * S::kVStride];
    __shared__ uint32_t s_row[kSub];

    const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
    const int split = blockIdx.x, kvh = blockIdx.y / n_qb, qb = blockIdx.y % n_qb, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    const int t0 = split * a.chunk;
    const int nt_total = min(a.chunk, len - t0);                 // <= 0: nothing of this split is valid

    RowInfo ri[kTilesPerWave];
    int vis[kTilesPerWave];                                      // tokens [0, vis) of the tier are visible to the row
    bf16x8 qop[kTilesPerWave][D / 32];
    float m[kTilesPerWave], l[kTilesPerWave];
    floatx4 acc[kTilesPerWave][DT];
#pragma unroll
    for (int rt = 0; rt < kTilesPerWave; ++rt) {
        ri[rt] = row_info<G>(a, b, kvh, qb * kRowsPerBlock + (w + kAWaves * rt) * 16 + n);
        vis[rt] = !ri[rt].valid ? 0 : a.causal_tail ? min(max(len - a.n_q + ri[rt].query + 1, 0), len) : len;
        load_q_tile<D>(a, ri[rt], g, qop[rt]);
        m[rt] = -INFINITY;
        l[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc[rt][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    StepLoader<D, true> ld;
    for (int sub0 = 0; sub0 < nt_total; sub0 += kSub) {
        const int nsub = min(kSub, nt_total - sub0);
        __syncthreads();                         // the previous table and stages are no longer in use
        const RowMap rows = make_row_map<false, kABlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0 + sub0, nsub, nullptr);
        const int steps = (nsub + kStepTokens - 1) / kStepTokens;
        ld.fetch(a.kv, rows, 0, nsub);
        for (int s = 0; s < steps; ++s) {
            const int buf = s & 1;
            ld.park(s_k[buf], s_v[buf]);
            if (s + 1 < steps) ld.fetch(a.kv, rows, s + 1, nsub);
            __syncthreads();

            // V^T operands of the step (shared by the wave's row tiles): 8 tokens of one output column
            bf16x8 vop[DT];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                uint32_t wd[4];
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    const uint32_t lo = *reinterpret_cast<const uint16_t *>(s_v[buf] + step_token(g, i) * S::kVStride + (dt * 16 + n) * 2);
                    const uint32_t hi = *reinterpret_cast<const uint16_t *>(s_v[buf] + step_token(g, i + 1) * S::kVStride + (dt * 16 + n) * 2);
                    wd[i / 2] = lo | (hi << 16);
                }
                vop[dt] = __builtin_bit_cast(bf16x8, make_uint4(wd[0], wd[1], wd[2], wd[3]));
            }

            const int step0 = t0 + sub0 + s * kStepTokens;       // tier position of the step's first token
            const int in_split = nsub - s * kStepTokens;         // tokens of the step that belong to this split
#pragma unroll
            for (int rt = 0; rt < kTilesPerWave; ++rt) {
                if (qb * kRowsPerBlock + (w + kAWaves * rt) * 16 >= a.n_q * G) continue;   // uniform over the wave
                float sv[8];
                tile_scores<D>(s_k[buf], qop[rt], a.sh.sm_scale, min(in_split, vis[rt] - step0), sv);
                float mx = sv[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
                mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
                mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                const float m_new = fmaxf(m[rt], mx);
                float p[8], ps = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = (m_new == -INFINITY) ? 0.f : __expf(sv[e] - m_new);   // masked scores give 0
                    ps += p[e];
                }
                ps += __shfl_xor(ps, 16, kWave);
                ps += __shfl_xor(ps, 32, kWave);
                const float corr = (m[rt] == -INFINITY) ? 0.f : __expf(m[rt] - m_new);
                l[rt] = l[rt] * corr + ps;
                m[rt] = m_new;
                if (__any(corr != 1.f)) {
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) acc[rt][dt] *= corr;
                }
                uint32_t hi[8], lo[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    hi[e] = bf16_rne(p[e]);
                    if (SPLIT_P) lo[e] = bf16_rne(p[e] - __uint_as_float(hi[e] << 16));
                }
                const bf16x8 ph = __builtin_bit_cast(bf16x8, make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16),
                                                                        hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16)));
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    acc[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[dt], ph, acc[rt][dt], 0, 0, 0);
                if (SPLIT_P) {
                    const bf16x8 pl = __builtin_bit_cast(bf16x8, make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16),
                                                                            lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)));
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
                        acc[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[dt], pl, acc[rt][dt], 0, 0, 0);
                }
            }
        }
    }

    // partial of every valid row: lane (n, g) holds output columns dt*16 + 4g .. +3 of row n
#pragma unroll
    for (int rt = 0; rt < kTilesPerWave; ++rt) {
        if (!ri[rt].valid) continue;
        const int64_t at = ri[rt].out_row * a.part.n_splits + split;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            *reinterpret_cast<float4 *>(a.part.o + at * D + dt * 16 + 4 * g) =
                make_float4(acc[rt][dt][0], acc[rt][dt][1], acc[rt][dt][2], acc[rt][dt][3]);
        if (g == 0) {
            a.part.m[at] = m[rt];
            a.part.l[at] = l[rt];
        }
    }
}

// Query-averaged softmax weights of a tier: a_out[b, h, t] = (1/N) sum_i e^{s_it - lse_i} over the queries i
// that see token t (lse_i is the tier's own log-sum-exp for query i), 0 beyond the length.
template <int D, int G>
__global__ __launch_bounds__(kABlock) void append_weights_kernel(AppendArgs a)
{
    using S = AStage<D>;
    __shared__ uint4 s_k[2][kStepTokens * S::kKStride];
    __shared__ uint32_t s_row[kSub];
    __shared__ float s_part[kAWaves][G][kStepTokens];
    __shared__ float s_out[G][kSub];

    const int chunk_id = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    const int t0 = chunk_id * a.chunk;                           // a.chunk <= kSub
    const int n_here = min(a.chunk, a.kv.cap - t0);              // entries of a_out this workgroup writes
    const int nsub = min(a.chunk, len - t0);                     // valid tokens among them
    for (int i = tid; i < G * kSub; i += kABlock) (&s_out[0][0])[i] = 0.f;

    if (nsub > 0) {
        __syncthreads();
        const RowMap rows = make_row_map<false, kABlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0, nsub, nullptr);
        const int steps = (nsub + kStepTokens - 1) / kStepTokens;
        const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
        StepLoader<D, false> ld;
        for (int qb = 0; qb < n_qb; ++qb) {
            RowInfo ri[kTilesPerWave];
            int vis[kTilesPerWave];
            float lse[kTilesPerWave];
            bf16x8 qop[kTilesPerWave][D / 32];
#pragma unroll
            for (int rt = 0; rt < kTilesPerWave; ++rt) {
                ri[rt] = row_info<G>(a, b, kvh, qb * kRowsPerBlock + (w + kAWaves * rt) * 16 + n);
                vis[rt] = !ri[rt].valid ? 0 : a.causal_tail ? min(max(len - a.n_q + ri[rt].query + 1, 0), len) : len;
                lse[rt] = ri[rt].valid ? a.lse[ri[rt].out_row] : -INFINITY;
                load_q_tile<D>(a, ri[rt], g, qop[rt]);
            }
            __syncthreads();                     // stages of the previous query block are no longer in use
            ld.fetch(a.kv, rows, 0, nsub);
            for (int s = 0; s < steps; ++s) {
                const int buf = s & 1;
                ld.park(s_k[buf], nullptr);
                if (s + 1 < steps) ld.fetch(a.kv, rows, s + 1, nsub);
                __syncthreads();
                const int step0 = t0 + s * kStepTokens, in_split = nsub - s * kStepTokens;
                float sum[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) sum[e] = 0.f;
#pragma unroll
                for (int rt = 0; rt < kTilesPerWave; ++rt) {
                    float sv[8];
                    tile_scores<D>(s_k[buf], qop[rt], a.sh.sm_scale, min(in_split, vis[rt] - step0), sv);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sum[e] += (lse[rt] == -INFINITY) ? 0.f : expf(sv[e] - lse[rt]);
                }
                // add the rows of the same head: columns n, n + G, n + 2G, ... of the 16-lane group
#pragma unroll
                for (int e = 0; e < 8; ++e) {
#pragma unroll
                    for (int off = G; off < 16; off <<= 1) sum[e] += __shfl_xor(sum[e], off, kWave);
                }
                if (n < G) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) s_part[w][n][16 * (e / 4) + 4 * g + (e % 4)] = sum[e];
                }
                __syncthreads();
                for (int i = tid; i < G * kStepTokens; i += kABlock) {
                    const int gh = i / kStepTokens, tok = i % kStepTokens;
                    float v = 0.f;
#pragma unroll
                    for (int ww = 0; ww < kAWaves; ++ww) v += s_part[ww][gh][tok];
                    s_out[gh][s * kStepTokens + tok] += v;       // one thread per entry: fixed order
                }
            }
        }
    }
    __syncthreads();
    const float inv_n = 1.f / (float)a.n_q;
    for (int i = tid; i < G * n_here; i += kABlock) {
        const int gh = i / n_here, j = i % n_here;
        a.a_out[((int64_t)b * a.sh.n_q_heads + kvh * G + gh) * a.kv.cap + t0 + j] = j < nsub ? s_out[gh][j] * inv_n : 0.f;
    }
}

template <int D, bool SPLIT_P>
hipError_t launch_attn_group(const AppendArgs &a, dim3 grid, hipStream_t s)
{
    switch (a.sh.group) {
    case 1: hipLaunchKernelGGL((append_attn_kernel<D, 1, SPLIT_P>), grid, dim3(kABlock), 0, s, a); break;
    case 2: hipLaunchKernelGGL((append_attn_kernel<D, 2, SPLIT_P>), grid, dim3(kABlock), 0, s, a); break;
    case 4: hipLaunchKernelGGL((append_attn_kernel<D, 4, SPLIT_P>), grid, dim3(kABlock), 0, s, a); break;
    case 8: hipLaunchKernelGGL((append_attn_kernel<D, 8, SPLIT_P>), grid, dim3(kABlock), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D>
hipError_t launch_weights_group(const AppendArgs &a, dim3 grid, hipStream_t s)
{
    switch (a.sh.group) {
    case 1: hipLaunchKernelGGL((append_weights_kernel<D, 1>), grid, dim3(kABlock), 0, s, a); break;
    case 2: hipLaunchKernelGGL((append_weights_kernel<D, 2>), grid, dim3(kABlock), 0, s, a); break;
    case 4: hipLaunchKernelGGL((append_weights_kernel<D, 4>), grid, dim3(kABlock), 0, s, a); break;
    case 8: hipLaunchKernelGGL((append_weights_kernel<D, 8>), grid, dim3(kABlock), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

#ifndef HGCA_APPEND_SPLIT_P
#define HGCA_APPEND_SPLIT_P 1
#endif

hipError_t launch_append_attn(int head_dim, const AppendArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.n_q == 0 || a.part.n_splits == 0) return hipSuccess;
    const int n_qb = (a.n_q * a.sh.group + kRowsPerBlock - 1) / kRowsPerBlock;
    dim3 grid(a.part.n_splits, a.sh.n_kv_heads * n_qb, a.sh.batch);
    constexpr bool kSplit = HGCA_APPEND_SPLIT_P != 0;
    if (head_dim == 64) return launch_attn_group<64, kSplit>(a, grid, s);
    if (head_dim == 128) return launch_attn_group<128, kSplit>(a, grid, s);
    return hipErrorInvalidValue;
}

hipError_t launch_append_weights(int head_dim, const AppendArgs &a, int n_chunks, hipStream_t s)
{
    if (a.sh.batch == 0 || n_chunks == 0) return hipSuccess;
    dim3 grid(n_chunks, a.sh.n_kv_heads, a.sh.batch);
    if (head_dim == 64) return launch_weights_group<64>(a, grid, s);
    if (head_dim == 128) return launch_weights_group<128>(a, grid, s);
    return hipErrorInvalidValue;
}

}  // namespace hgca
