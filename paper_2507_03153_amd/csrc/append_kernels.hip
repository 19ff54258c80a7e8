// Append stage: N queries per sequence attend to one KV tier (Sec. 2.1: S = Q K^T, A = softmax(S),
// O = A V with Q in R^{h x N x d}; Alg. 2, append branch).  bf16 inputs, both contractions on
// v_mfma_f32_16x16x32_bf16.
//
// Work unit: one workgroup = one split of the tokens of one (sequence, KV head) and up to 128 query
// rows (a row = one query x one head of the GQA group, query-major).  Each of the eight waves owns
// one 16-row tile, so nothing is reduced across waves; all 512 threads stage the K and V rows of a
// 64-token step into LDS with coalesced 16-byte loads.  The next step's loads are in flight during a
// step's arithmetic (registers, parked into a double-buffered LDS stage, one barrier per step); two
// workgroups share a CU, so 64 KB per CU are on their way from HBM while 16 waves do arithmetic.
// A step is 64 tokens rather than 32 because the softmax of a step is one dependent chain (scores,
// row maximum, exponentials, row sum, rounding, second contraction): four score tiles per chain give
// the wave independent work to overlap it with.
//
// Orientation (per 16-row tile, per step):
//   S^T[token, row]  = K[token, :] . Q[row, :]        A = K tile (LDS, padded rows), B = Q (registers)
//   O^T[dcol, row]  += V^T[dcol, token] . P^T[token, row]   A = V^T (LDS transpose reads of the rows), B = P
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

constexpr int kABlock = 512;
constexpr int kAWaves = kABlock / kWave;
constexpr int kStepBlocks = 2;                   // 32-token contraction blocks per step
constexpr int kStepTokens = 32 * kStepBlocks;
constexpr int kRowsPerBlock = 128;               // query rows per workgroup = 8 tiles of 16, one per wave
static_assert(kRowsPerBlock == 16 * kAWaves, "one row tile per wave");
constexpr int kSub = kMaxChunk;                  // tokens per refill of the row table

template <int D> struct AStage {
    static constexpr int kPieces = D / 8;                        // 16-byte pieces per row
    static constexpr int kKStride = kPieces + 1;                 // K row stride in uint4 (conflict-free b128 reads)
    static constexpr int kVStride = D * 2 + 32;                  // V row stride in bytes: 4 consecutive rows x 32 bytes
                                                                 // cover all banks (transpose reads of a lane group)
    static constexpr int kTotal = kStepTokens * kPieces;         // 16-byte pieces of a step, per tensor
    static constexpr int kLoads = (kTotal + kABlock - 1) / kABlock;  // loads per thread, step and tensor
};

// The value of the lane ROT places further on in the same row of 16 lanes (DPP row_ror).
template <int ROT>
__device__ __forceinline__ float row_rotate(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + ROT, 0xf, 0xf, true));
}

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

// Stages the K (and V) rows of a step: global -> registers -> LDS, one step ahead.
template <int D, bool WITH_V>
struct StepLoader {
    using S = AStage<D>;
    static constexpr size_t ROW_BYTES = D * 2;
    uint4 kr[S::kLoads], vr[S::kLoads];

    __device__ __forceinline__ void fetch(const KvDev &kv, const RowMap &rows, int step, int nsub) {
#pragma unroll
        for (int u = 0; u < S::kLoads; ++u) {
            const int p = threadIdx.x + kABlock * u, trow = p / S::kPieces, piece = p % S::kPieces;
            if (p >= S::kTotal) break;
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
            if (p >= S::kTotal) break;
            s_k[trow * S::kKStride + piece] = kr[u];
            if (WITH_V) *reinterpret_cast<uint4 *>(s_v + trow * S::kVStride + 16 * piece) = vr[u];
        }
    }
};

// Raw scores <q, k> (no softmax scale yet) of one 16-row tile for the step's tokens: sv[8*kb + 4*tt + r] belongs
// to step token 32*kb + 16*tt + 4*g + r and query row lane % 16.  With MASK, tokens at or beyond `limit` (counted
// from the step's first token) read -inf.
template <int D, bool MASK>
__device__ __forceinline__ void tile_scores(const uint4 *s_k, const bf16x8 (&qop)[D / 32], int limit,
                                            float (&sv)[8 * kStepBlocks])
{
    using S = AStage<D>;
    const int lane = threadIdx.x % kWave, n = lane % 16, g = lane / 16;
#pragma unroll
    for (int t = 0; t < 2 * kStepBlocks; ++t) {  // 16-token tiles of the step
        floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            const uint4 ka = s_k[(t * 16 + n) * S::kKStride + 4 * kk + g];
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qop[kk], c, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sv[4 * t + r] = (!MASK || 16 * t + 4 * g + r < limit) ? c[r] : -INFINITY;
    }
}

// Runs `body(stage, step)` for every step of a sub-chunk with the next step's loads in flight.  A stage
// written in step s is read in step s and rewritten in step s + 2; the barrier of step s + 1 lies between,
// so one barrier per step orders everything.
template <int D, bool WITH_V, typename Body>
__device__ __forceinline__ void for_each_step(const KvDev &kv, const RowMap &rows, int nsub, uint4 (*s_k)[kStepTokens * AStage<D>::kKStride],
                                              char (*s_v)[kStepTokens * AStage<D>::kVStride], Body body)
{
    const int steps = (nsub + kStepTokens - 1) / kStepTokens;
    StepLoader<D, WITH_V> ld;
    ld.fetch(kv, rows, 0, nsub);
    for (int s = 0; s < steps; ++s) {
        ld.park(s_k[s & 1], WITH_V ? s_v[s & 1] : nullptr);
        if (s + 1 < steps) ld.fetch(kv, rows, s + 1, nsub);
        __syncthreads();
        body(s & 1, s);
    }
}

template <int D, int G, bool SPLIT_P>
__global__ __launch_bounds__(kABlock, 4) void append_attn_kernel(AppendArgs a)
{
    using S = AStage<D>;
    constexpr int DT = D / 16;
    constexpr float kLog2e = 1.4426950408889634f;
    __shared__ uint4 s_k[2][kStepTokens * S::kKStride];
    __shared__ __attribute__((aligned(16))) char s_v[2][kStepTokens * S::kVStride];
    __shared__ uint32_t s_row[kSub];

    const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
    const int split = blockIdx.x, kvh = blockIdx.y / n_qb, qb = blockIdx.y % n_qb, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    const int t0 = split * a.chunk;
    const int nt_total = min(a.chunk, len - t0);                 // <= 0: nothing of this split is valid

    const int tile_row0 = qb * kRowsPerBlock + w * 16;           // first row of the wave's tile
    const bool tile_live = tile_row0 < a.n_q * G;                // uniform over the wave
    const RowInfo ri = row_info<G>(a, b, kvh, tile_row0 + n);
    // tokens [0, vis) of the tier are visible to the row
    const int vis = !ri.valid ? 0 : a.causal_tail ? min(max(len - a.n_q + ri.query + 1, 0), len) : len;
    int vis_min = vis;                           // over the rows of the tile: steps below it need no mask
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) vis_min = min(vis_min, __shfl_xor(vis_min, off, kWave));
    bf16x8 qop[D / 32];
    load_q_tile<D>(a, ri, g, qop);
    // The running maximum m is kept on the RAW scores (the softmax scale is positive, so the order is the same) and
    // the scale, in units of ln 2, is applied inside the exponent: e^{scale (s - m)} = 2^{fma(s, scale2, -m scale2)},
    // one fused multiply-add and one bare v_exp_f32 per score.
    const float scale2 = a.sh.sm_scale * kLog2e;
    float m = -INFINITY, l = 0.f;
    floatx4 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};

    // a paged tier needs a row table in LDS, refilled every kSub tokens (which drains the load pipeline);
    // a contiguous tier is plain arithmetic and takes the whole split in one pass
    const int sub_len = a.kv.block_table ? kSub : max(nt_total, 1);
    for (int sub0 = 0; sub0 < nt_total; sub0 += sub_len) {
        const int nsub = min(sub_len, nt_total - sub0);
        __syncthreads();                         // the previous table and stages are no longer in use
        const RowMap rows = make_row_map<false, kABlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0 + sub0, nsub, nullptr);
        for_each_step<D, true>(a.kv, rows, nsub, s_k, s_v, [&](int buf, int s) {
            if (!tile_live) return;
            const int step0 = t0 + sub0 + s * kStepTokens;       // tier position of the step's first token
            const int in_split = nsub - s * kStepTokens;         // tokens of the step that belong to this split
            float sv[8 * kStepBlocks];
            if (min(in_split, vis_min - step0) >= kStepTokens)   // uniform over the wave: every token visible to every row
                tile_scores<D, false>(s_k[buf], qop, 0, sv);
            else
                tile_scores<D, true>(s_k[buf], qop, min(in_split, vis - step0), sv);
            float mx = sv[0];
#pragma unroll
            for (int e = 1; e < 8 * kStepBlocks; ++e) mx = fmaxf(mx, sv[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m, mx);
            // a row that has seen nothing yet keeps m = -inf: shift by 0 then, every exponent is -inf and gives 0
            const float shift = (m_new == -INFINITY) ? 0.f : -m_new * scale2;
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8 * kStepBlocks; ++e) {          // sv becomes the probabilities; masked scores give 0
                sv[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], scale2, shift));
                ps += sv[e];
            }
            ps += __shfl_xor(ps, 16, kWave);
            ps += __shfl_xor(ps, 32, kWave);
            const float corr = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(fmaf(m, scale2, shift));
            l = l * corr + ps;
            m = m_new;
            if (__any(corr != 1.f)) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc[dt] *= corr;
            }
#pragma unroll
            for (int kb = 0; kb < kStepBlocks; ++kb) {
                bf16x8 ph, pl;                   // round to nearest even; the low part carries the rounding error
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    ph[e] = (__bf16)sv[8 * kb + e];
                    pl[e] = SPLIT_P ? (__bf16)(sv[8 * kb + e] - (float)ph[e]) : (__bf16)0.f;
                }
                // O^T += V^T P^T, one 16-column tile of the output at a time.  The V^T operand (8 tokens of one column
                // per lane) comes from two transpose reads: lane j of a group points at columns 4(j%4).. of the row of
                // contraction index j/4 (first read) and 4 + j/4 (second read).
                const char *v_lo = s_v[buf] + (32 * kb + block_token(g, n / 4)) * S::kVStride + 8 * (n % 4);
                const char *v_hi = s_v[buf] + (32 * kb + block_token(g, 4 + n / 4)) * S::kVStride + 8 * (n % 4);
                // column tiles in groups of kPvGroup: the group's high-part products first, then its low-part ones, so
                // that two MFMAs on the same accumulator are kPvGroup instructions apart
                constexpr int kPvGroup = 4;
#pragma unroll
                for (int dt0 = 0; dt0 < DT; dt0 += kPvGroup) {
                    bf16x8 vop[kPvGroup];
#pragma unroll
                    for (int u = 0; u < kPvGroup; ++u) {
                        const short4v a0 = lds_read_tr16(v_lo + 32 * (dt0 + u)), a1 = lds_read_tr16(v_hi + 32 * (dt0 + u));
                        const short8v both = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                        vop[u] = __builtin_bit_cast(bf16x8, both);
                    }
#pragma unroll
                    for (int u = 0; u < kPvGroup; ++u)
                        acc[dt0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[u], ph, acc[dt0 + u], 0, 0, 0);
                    if (SPLIT_P) {
#pragma unroll
                        for (int u = 0; u < kPvGroup; ++u)
                            acc[dt0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[u], pl, acc[dt0 + u], 0, 0, 0);
                    }
                }
            }
        });
    }

    // partial of every valid row: lane (n, g) holds output columns dt*16 + 4g .. +3 of row n
    if (ri.valid) {
        const int64_t at = ri.out_row * a.part.n_splits + split;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            *reinterpret_cast<float4 *>(a.part.o + at * D + dt * 16 + 4 * g) =
                make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]);
        if (g == 0) {
            a.part.m[at] = m * a.sh.sm_scale;    // the maximum of the scaled scores (-inf stays -inf)
            a.part.l[at] = l;
        }
    }
}

// Query-averaged softmax weights of a tier: a_out[b, h, t] = (1/N) sum_i e^{s_it - lse_i} over the queries i
// that see token t (lse_i is the tier's own log-sum-exp for query i), 0 beyond the length.  One workgroup
// owns a_out[b, heads of kvh, t0 .. t0 + chunk): every step the waves' sums go through LDS to one thread
// per entry, which writes (first block of 128 query rows) or adds to (further blocks) the entry.
template <int D, int G>
__global__ __launch_bounds__(kABlock) void append_weights_kernel(AppendArgs a)
{
    using S = AStage<D>;
    __shared__ uint4 s_k[2][kStepTokens * S::kKStride];
    __shared__ uint32_t s_row[kSub];
    __shared__ float s_part[2][kAWaves][G][kStepTokens];         // per stage: read after the next step's barrier

    const int chunk_id = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    const int t0 = chunk_id * a.chunk;
    const int n_here = min(a.chunk, a.kv.cap - t0);              // entries of a_out this workgroup writes
    const int nt_total = min(a.chunk, len - t0);                 // valid tokens among them (may be <= 0)
    const float inv_n = 1.f / (float)a.n_q;
    constexpr float kLog2e = 1.4426950408889634f;
    const float scale2 = a.sh.sm_scale * kLog2e;
    float *out = a.a_out + ((int64_t)b * a.sh.n_q_heads + kvh * G) * a.kv.cap + t0;

    const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
    const int sub_len = a.kv.block_table ? kSub : max(nt_total, 1);
    for (int qb = 0; qb < n_qb && nt_total > 0; ++qb) {
        const RowInfo ri = row_info<G>(a, b, kvh, qb * kRowsPerBlock + w * 16 + n);
        const int vis = !ri.valid ? 0 : a.causal_tail ? min(max(len - a.n_q + ri.query + 1, 0), len) : len;
        // minus the row's lse in units of ln 2; a row that sees nothing has lse = -inf and only masked (-inf) scores,
        // which a shift of 0 turns into weights 0
        const float row_lse = ri.valid ? a.lse[ri.out_row] : -INFINITY;
        const float neg_lse2 = (row_lse == -INFINITY) ? 0.f : -row_lse * kLog2e;
        bf16x8 qop[D / 32];
        load_q_tile<D>(a, ri, g, qop);
        for (int sub0 = 0; sub0 < nt_total; sub0 += sub_len) {
            const int nsub = min(sub_len, nt_total - sub0);
            __syncthreads();                     // table, stages and sums of the previous pass are no longer in use
            const RowMap rows = make_row_map<false, kABlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0 + sub0, nsub, nullptr);
            int pending = -1;                    // step whose per-wave sums wait in s_part[pending & 1]
            auto fold = [&](int step) {          // one thread per entry, waves added in a fixed order
                for (int i = tid; i < G * kStepTokens; i += kABlock) {
                    const int gh = i / kStepTokens, tok = sub0 + step * kStepTokens + i % kStepTokens;
                    if (tok >= nt_total) continue;
                    float v = 0.f;
#pragma unroll
                    for (int ww = 0; ww < kAWaves; ++ww) v += s_part[step & 1][ww][gh][i % kStepTokens];
                    float *dst = out + (int64_t)gh * a.kv.cap + tok;
                    *dst = qb == 0 ? v * inv_n : fmaf(v, inv_n, *dst);
                }
            };
            for_each_step<D, false>(a.kv, rows, nsub, s_k, static_cast<char (*)[kStepTokens * S::kVStride]>(nullptr),
                                    [&](int buf, int s) {
                if (pending >= 0) fold(pending);                 // written before the barrier that preceded this call
                float sv[8 * kStepBlocks];
                const int step0 = sub0 + s * kStepTokens;
                tile_scores<D, true>(s_k[buf], qop, min(nsub - s * kStepTokens, vis - (t0 + step0)), sv);
#pragma unroll
                for (int e = 0; e < 8 * kStepBlocks; ++e) {
                    float x = __builtin_amdgcn_exp2f(fmaf(sv[e], scale2, neg_lse2));
                    // add the rows of the same head: columns n, n + G, n + 2G, ... of the 16-lane row, by rotating
                    // the row (DPP row_ror) by 8, 4, ... G lanes
                    if (G <= 8) x += row_rotate<8>(x);
                    if (G <= 4) x += row_rotate<4>(x);
                    if (G <= 2) x += row_rotate<2>(x);
                    if (G <= 1) x += row_rotate<1>(x);
                    if (n < G) s_part[s & 1][w][n][16 * (e / 4) + 4 * g + (e % 4)] = x;
                }
                pending = s;
            });
            __syncthreads();
            if (pending >= 0) fold(pending);
        }
    }
    // entries beyond the sequence's length
    for (int i = tid; i < G * n_here; i += kABlock) {
        const int gh = i / n_here, j = i % n_here;
        if (j >= nt_total) out[(int64_t)gh * a.kv.cap + j] = 0.f;
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
