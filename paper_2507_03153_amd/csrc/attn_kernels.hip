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
#include "hgca_launch.hpp"
#include "row_map.hpp"

namespace hgca {

namespace {

// kGatherScored: scores are given; kGatherGroup: one index list per KV head, shared by the NH heads of its group
enum Mode { kDense = 0, kGather = 1, kScores = 2, kGatherScored = 3, kGatherGroup = 4 };

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
#ifndef HGCA_UNROLL
#define HGCA_UNROLL 4
#endif
constexpr int kUnroll = HGCA_UNROLL;   // 16-byte loads a lane keeps in flight in the K / V passes


struct KernelArgs {
    ShapeDev sh;
    const char *q;
    KvDev kv;
    const int32_t *idx;
    const int32_t *cnt;
    const float *sel_scores;
    int32_t k_max;
    int32_t chunk;
    Partials part;
    float *scores;
    int32_t group_max;     // score pass: write one row per KV head, the maximum over the group's heads
};

// ---- pieces shared by all split kernels ---------------------------------------------------

template <int D, int NH>
__device__ __forceinline__ void write_empty_partial(const Partials &part, int64_t bh0, int split)
{
    for (int i = threadIdx.x; i < NH * D; i += kBlock) {
        const int g = i / D, col = i % D;
        part.o[((bh0 + g) * part.n_splits + split) * D + col] = 0.f;
    }
    if (threadIdx.x < NH) {
        part.m[(bh0 + threadIdx.x) * part.n_splits + split] = -INFINITY;
        part.l[(bh0 + threadIdx.x) * part.n_splits + split] = 0.f;
    }
}

// s_p[g][0..nt) holds scores on entry and weights e^{s-m} on exit; one wave per head.
template <int NH>
__device__ __forceinline__ void split_softmax(float (*s_p)[kMaxChunk], float *s_m, float *s_l, int nt)
{
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
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
}

// o[g][:] = sum_j p[g][j] v_j over the split, reduced over the workgroup and written as a partial.
template <typename T, int D, int NH, bool GATHER>
__device__ __forceinline__ void value_pass(const KernelArgs &a, float (*s_p)[kMaxChunk],
                                           float (*s_red)[NH][D], const float *s_m, const float *s_l,
                                           int64_t bh0, int split, int nt, const RowMap &rows)
{
    constexpr int EPL = Elem<T>::kPerLoad;       // elements per lane per load
    constexpr int LPR = D / EPL;                 // lanes per row
    constexpr int RPW = kWave / LPR;             // rows per wave per load
    constexpr int RPI = kWaves * RPW;            // rows per workgroup iteration
    constexpr size_t ROW_BYTES = D * sizeof(T);
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int r = lane / LPR, c = lane % LPR;

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
            vr[u] = load16_stream(a.kv.v + rows(j) * ROW_BYTES + c * 16);
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

// Scaled scores of the split to a.scores[b, h, t0 .. t0+nt) for the NH heads of the workgroup.
template <int NH>
__device__ __forceinline__ void store_split_scores(const KernelArgs &a, const float (*s_p)[kMaxChunk], int64_t bh0,
                                                   int t0, int nt)
{
    if (a.group_max) {                           // one row per KV head: row index bh0 / NH (bh0 is the group's first head)
        for (int j = threadIdx.x; j < nt; j += kBlock) {
            float v = s_p[0][j];
#pragma unroll
            for (int g = 1; g < NH; ++g) v = fmaxf(v, s_p[g][j]);
            a.scores[(bh0 / NH) * (int64_t)a.kv.cap + t0 + j] = v;
        }
        return;
    }
    for (int i = threadIdx.x; i < NH * nt; i += kBlock) {
        const int g = i / nt, j = i % nt;
        a.scores[(bh0 + g) * (int64_t)a.kv.cap + t0 + j] = s_p[g][j];
    }
}

// ---- VALU path -----------------------------------------------------------------------------

template <typename T, int D, int NH, int MODE>
__global__ __launch_bounds__(kBlock) void attn_split_kernel(KernelArgs a)
{
    constexpr int EPL = Elem<T>::kPerLoad;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int RPI = kWaves * RPW;
    constexpr size_t ROW_BYTES = D * sizeof(T);

    __shared__ float s_p[NH][kMaxChunk];         // scores of the split, then weights
    __shared__ uint32_t s_row[kMaxChunk];
    __shared__ float s_red[kWaves][NH][D];
    __shared__ float s_m[NH], s_l[NH];

    const int split = blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
    const int Hq = a.sh.n_q_heads, Hkv = a.sh.n_kv_heads;
    constexpr bool GATHER = MODE == kGather || MODE == kGatherScored || MODE == kGatherGroup;
    constexpr bool PER_HEAD_LIST = MODE == kGather || MODE == kGatherScored;
    const int kvh = PER_HEAD_LIST ? unit / a.sh.group : unit;
    const int h0 = PER_HEAD_LIST ? unit : unit * NH;             // first of the NH heads handled
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int r = lane / LPR, c = lane % LPR;

    const int64_t bh0 = (int64_t)b * Hq + h0;
    const int64_t list = PER_HEAD_LIST ? bh0 : (int64_t)b * Hkv + unit;      // row of idx / cnt
    const int n = GATHER ? (a.kv.cap > 0 ? min(a.cnt[list], a.k_max) : 0) : tier_len(a.kv, b);
    const int t0 = split * a.chunk;

    if (t0 >= n) {                               // empty split (uniform over the workgroup)
        if (MODE != kScores) write_empty_partial<D, NH>(a.part, bh0, split);
        return;
    }
    const int nt = min(a.chunk, n - t0);         // 1 .. chunk tokens in this split
    if (MODE == kGatherScored) {                 // the caller already holds the scores of the listed entries
        const float *given = a.sel_scores + bh0 * a.k_max + t0;
        for (int j = tid; j < nt; j += kBlock) s_p[0][j] = given[j];
    }
    const RowMap rows = make_row_map<GATHER, kBlock>(s_row, a.kv, Hkv, b, kvh, t0, nt,
                                                     GATHER ? a.idx + list * a.k_max + t0 : nullptr);
    float qf[NH][EPL];
    if (MODE != kGatherScored) {
#pragma unroll
        for (int g = 0; g < NH; ++g)
            Elem<T>::expand(load16(a.q + ((bh0 + g) * D + c * EPL) * (int64_t)sizeof(T)), qf[g]);
    }

    // K pass: scores of the split into LDS
    for (int base = 0; MODE != kGatherScored && base < nt; base += RPI * kUnroll) {
        uint4 kr[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = min(base + u * RPI + w * RPW + r, nt - 1);
            kr[u] = load16_stream(a.kv.k + rows(j) * ROW_BYTES + c * 16);
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

    if (MODE == kScores || (MODE == kDense && a.scores)) store_split_scores<NH>(a, s_p, bh0, t0, nt);
    if (MODE == kScores) return;
    if (MODE == kDense && a.scores) __syncthreads();   // the softmax below overwrites the scores other waves are still storing

    split_softmax<NH>(s_p, s_m, s_l, nt);
    __syncthreads();
    value_pass<T, D, NH, GATHER>(a, s_p, s_red, s_m, s_l, bh0, split, nt, rows);
}

// ---- MFMA path (bf16 K/V, dense over a tier) -------------------------------------------------

// B operand of the score MFMAs: column n = lane % 16 is query head h0 + n of the group (zero beyond
// the group); k-slice kk holds q[32*kk + 8*(lane/16) .. +8), the same d-slice the A operand takes.
template <int D, int G>
__device__ __forceinline__ void load_q_operand(const char *q, int64_t bh0, bf16x8 (&qb)[D / 32])
{
    const int lane = threadIdx.x % kWave, n = lane % 16, g = lane / 16;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        uint4 r = make_uint4(0u, 0u, 0u, 0u);
        if (n < G) r = load16(q + ((bh0 + n) * D + 32 * kk + 8 * g) * 2);
        qb[kk] = __builtin_bit_cast(bf16x8, r);
    }
}

// K tiles reach the MFMA through LDS: a wave loads a 16-token tile with fully coalesced 16-byte
// loads (consecutive lanes take consecutive 16-byte pieces of a row), parks it in its own LDS stage
// with one 16-byte pad per row (conflict-free b128 reads), and reads it back in A-operand layout.
template <int D> struct Stage {
    static constexpr int kPieces = D / 8;                    // 16-byte pieces per K row
    static constexpr int kRowStride = kPieces + 1;           // in uint4, padded
    static constexpr int kRowsPerLoad = kWave / kPieces;     // rows one load instruction covers
    static constexpr int kLoads = 16 / kRowsPerLoad;         // load instructions per tile
    static constexpr int kWaveVecs = 16 * kRowStride;        // uint4 per wave
};

// Scaled scores of tokens [t0, t0+nt) of (b, kvh) for the G heads of the group, written to
// s_sc[n][j] (n < G, j < nt rounded up to 16; entries at j >= nt are finite filler).
template <int D, int G, int LD, int NW = kWaves>
__device__ __forceinline__ void mfma_scores(const KernelArgs &a, uint4 *stage, float (*s_sc)[LD], int64_t bh0,
                                            int nt, const RowMap &rows)
{
    using S = Stage<D>;
    constexpr size_t ROW_BYTES = D * 2;
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int lrow = lane / S::kPieces, piece = lane % S::kPieces;   // role while loading
    const int row = lane % 16, g = lane / 16;                        // role as A operand / C result
    uint4 *st = stage + w * S::kWaveVecs;
    bf16x8 qb[D / 32];
    load_q_operand<D, G>(a.q, bh0, qb);

    const int n_tiles = (nt + 15) / 16;
    auto load_tile = [&](int ti, uint4 (&kr)[S::kLoads]) {
#pragma unroll
        for (int i = 0; i < S::kLoads; ++i) {
            const int j = min(ti * 16 + i * S::kRowsPerLoad + lrow, nt - 1);
            kr[i] = load16_stream(a.kv.k + rows(j) * ROW_BYTES + 16 * piece);
        }
    };
    // the next tile's loads are issued before the current tile goes through LDS and the MFMAs
    uint4 kr[S::kLoads], kr_next[S::kLoads];
    if (w < n_tiles) load_tile(w, kr);
    for (int ti = w; ti < n_tiles; ti += NW) {
        const bool more = ti + NW < n_tiles;
        if (more) load_tile(ti + NW, kr_next);
#pragma unroll
        for (int i = 0; i < S::kLoads; ++i) st[(i * S::kRowsPerLoad + lrow) * S::kRowStride + piece] = kr[i];
        __builtin_amdgcn_wave_barrier();         // same wave writes and reads its stage; LDS keeps wave order
        floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            const uint4 ka = st[row * S::kRowStride + 4 * kk + g];
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qb[kk], c, 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
        if (row < G) {                           // C layout: column n = row, tokens 4*g .. 4*g+3 of the tile
            const float sc = a.sh.sm_scale;
            *reinterpret_cast<float4 *>(&s_sc[row][ti * 16 + 4 * g]) =
                make_float4(c[0] * sc, c[1] * sc, c[2] * sc, c[3] * sc);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < S::kLoads; ++i) kr[i] = kr_next[i];
        }
    }
}

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
            __builtin_nontemporal_store(vv, reinterpret_cast<floatx4 *>(o));
        } else {
            if (j < nt) o[0] = v.x;
            if (j + 1 < nt) o[1] = v.y;
            if (j + 2 < nt) o[2] = v.z;
            if (j + 3 < nt) o[3] = v.w;
        }
    }
}

// Heads per group from which the V pass of the dense kernel runs on the matrix cores.  With 8 heads the VALU pass
// (G fused multiply-adds per loaded element) is bound by instruction issue (2.8 TB/s measured, 3.6 with MFMA);
// with 4 heads and fewer the VALU pass keeps up with HBM and needs less LDS (measured 31.2 against 32.3 us on C2).
#ifndef HGCA_DENSE_PV_MFMA_FROM
#define HGCA_DENSE_PV_MFMA_FROM 8
#endif
constexpr int kPvPad = 32;                       // bytes of padding per V row in the stage (conflict-free transpose reads)

// V pass on the matrix cores: O^T[dcol, head] += V^T[dcol, token] . P^T[token, head] in 32-token blocks, one wave
// per block.  The block's V rows are parked in a wave-private LDS stage as loaded (row-major) and come back
// through transpose reads as the A operand; the weights of the block (fp32 in s_p) are rounded to a high and a
// low bf16 part for the B operand (column = head, zero beyond the group).
template <int D, int G>
__device__ __forceinline__ void value_pass_mfma(const KernelArgs &a, float (*s_p)[kMaxChunk], char *stage,
                                                float (*s_red)[G][D], const float *s_m, const float *s_l, int64_t bh0,
                                                int split, int nt, const RowMap &rows)
{
    constexpr int DT = D / 16, PIECES = D / 8, VS = D * 2 + kPvPad, LOADS = 32 * PIECES / kWave;
    constexpr size_t ROW_BYTES = D * 2;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    char *st = stage + w * (32 * VS);
    floatx4 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int n_blocks = (nt + 31) / 32;
    auto load_block = [&](int blk, uint4 (&vr)[LOADS]) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int p = lane + kWave * u, trow = p / PIECES, piece = p % PIECES;
            vr[u] = load16_stream(a.kv.v + rows(min(blk * 32 + trow, nt - 1)) * ROW_BYTES + 16 * piece);
        }
    };
    uint4 vr[LOADS];
    if (w < n_blocks) load_block(w, vr);
    for (int blk = w; blk < n_blocks; blk += kWaves) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int p = lane + kWave * u, trow = p / PIECES, piece = p % PIECES;
            *reinterpret_cast<uint4 *>(st + trow * VS + 16 * piece) = vr[u];
        }
        if (blk + kWaves < n_blocks) load_block(blk + kWaves, vr);
        __builtin_amdgcn_wave_barrier();
        bf16x8 ph, pl;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = blk * 32 + block_token(g, i);
            const float p = (n < G && j < nt) ? s_p[n < G ? n : 0][j] : 0.f;
            ph[i] = (__bf16)p;
            pl[i] = (__bf16)(p - (float)ph[i]);
        }
        const char *v_lo = st + block_token(g, n / 4) * VS + 8 * (n % 4);
        const char *v_hi = st + block_token(g, 4 + n / 4) * VS + 8 * (n % 4);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const short4v a0 = lds_read_tr16(v_lo + 32 * dt), a1 = lds_read_tr16(v_hi + 32 * dt);
            const short8v both = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
            const bf16x8 vop = __builtin_bit_cast(bf16x8, both);
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, ph, acc[dt], 0, 0, 0);
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pl, acc[dt], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();                             // every wave is done with its stage: the reduction reuses the space
    if (n < G) {                                 // lane (head n, group g) holds output columns dt*16 + 4g .. +3
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            *reinterpret_cast<float4 *>(&s_red[w][n][dt * 16 + 4 * g]) =
                make_float4(acc[dt][0], acc[dt][1], acc[dt][2], acc[dt][3]);
    }
    __syncthreads();
    for (int i = tid; i < G * D; i += kBlock) {
        const int gg = i / D, col = i % D;
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) v += s_red[ww][gg][col];
        a.part.o[((bh0 + gg) * a.part.n_splits + split) * D + col] = v;
    }
    if (tid < G) {
        a.part.m[(bh0 + tid) * a.part.n_splits + split] = s_m[tid];
        a.part.l[(bh0 + tid) * a.part.n_splits + split] = s_l[tid];
    }
}

template <int D, int G>
__global__ __launch_bounds__(kBlock) void dense_attn_mfma_kernel(KernelArgs a)
{
    // the K stage is dead once the scores are in s_p; the V stage and the output reduction reuse its space
    constexpr int kStageBytes = kWaves * Stage<D>::kWaveVecs * 16;
    constexpr bool kPvMfma = G >= HGCA_DENSE_PV_MFMA_FROM;
    constexpr int kVStageBytes = kPvMfma ? kWaves * 32 * (D * 2 + kPvPad) : 0;
    constexpr int kRedBytes = kWaves * G * D * 4 + kVStageBytes;
    constexpr int kBufBytes = kStageBytes > kRedBytes ? kStageBytes : kRedBytes;
    __shared__ __attribute__((aligned(16))) char s_buf[kBufBytes];
    __shared__ __attribute__((aligned(16))) float s_p[G][kMaxChunk];
    __shared__ float s_m[G], s_l[G];
    __shared__ uint32_t s_row[kMaxChunk];

    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int64_t bh0 = (int64_t)b * a.sh.n_q_heads + (int64_t)kvh * G;
    const int n = tier_len(a.kv, b);
    const int t0 = split * a.chunk;
    if (t0 >= n) {
        write_empty_partial<D, G>(a.part, bh0, split);
        return;
    }
    const int nt = min(a.chunk, n - t0);
    const RowMap rows = make_row_map<false, kBlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0, nt, nullptr);
    mfma_scores<D, G, kMaxChunk>(a, reinterpret_cast<uint4 *>(s_buf), s_p, bh0, nt, rows);
    __syncthreads();
    if (a.scores) {                              // uniform over the workgroup
        store_split_scores<G>(a, s_p, bh0, t0, nt);
        __syncthreads();                         // the softmax below overwrites the scores other waves are still storing
    }
    split_softmax<G>(s_p, s_m, s_l, nt);
    __syncthreads();
    if (kPvMfma)                                 // V stage first, reduction area behind it
        value_pass_mfma<D, G>(a, s_p, s_buf, reinterpret_cast<float (*)[G][D]>(s_buf + kVStageBytes), s_m, s_l, bh0, split,
                              nt, rows);
    else
        value_pass<bf16_t, D, G, false>(a, s_p, reinterpret_cast<float (*)[G][D]>(s_buf), s_m, s_l, bh0, split, nt, rows);
}

// ---- combine and merge ------------------------------------------------------------------------------

// Folds split partials of one (b, h) row: M = max m_s, L = sum l_s e^{m_s-M}, O = sum o_s e^{m_s-M} / L,
// lse = M + ln L.  The splits may come from two partial sets (p and q): folding the splits of the dense
// window part and of the sparse part in one go is merge_state applied to all of them at once
// (the fusion is associative).  Thread (sg, c4) sums the splits sg, sg+SG, ... of four adjacent columns;
// the SG groups are then added through LDS.
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(kBlock) void combine_kernel(Partials p, Partials q, void *o, float *lse, float *lse_p)
{
    constexpr int C4 = D / 4;                    // threads across the columns (one float4 each)
    constexpr int SG = kBlock / C4;              // split groups
    __shared__ float4 s_acc[SG][C4];
    __shared__ float s_L[SG];

    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x, sg = tid / C4, c4 = tid % C4;
    const int np = p.n_splits, n = np + q.n_splits;
    auto m_of = [&](int s) { return s < np ? p.m[row * np + s] : q.m[row * q.n_splits + (s - np)]; };
    auto l_of = [&](int s) { return s < np ? p.l[row * np + s] : q.l[row * q.n_splits + (s - np)]; };
    auto o_of = [&](int s) {
        const float *base = s < np ? p.o + (row * np + s) * D : q.o + (row * q.n_splits + (s - np)) * D;
        return *reinterpret_cast<const float4 *>(base + 4 * c4);
    };
    // the maximum over all splits: one split per thread, then over the workgroup (a loop over the splits in every
    // thread would be a chain of dependent round trips to memory)
    __shared__ float s_M[kWaves];
    float M = -INFINITY;
    for (int s = tid; s < n; s += kBlock) M = fmaxf(M, m_of(s));
    M = wave_max(M);
    if (tid % kWave == 0) s_M[tid / kWave] = M;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, s_M[w]);
    float L = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (M != -INFINITY) {                        // else every split is empty (uniform over the workgroup)
        for (int s = sg; s < n; s += SG) {
            const float wgt = expf(m_of(s) - M); // 0 for empty splits (m = -inf)
            const float4 v = o_of(s);
            L = fmaf(l_of(s), wgt, L);
            acc.x = fmaf(v.x, wgt, acc.x); acc.y = fmaf(v.y, wgt, acc.y);
            acc.z = fmaf(v.z, wgt, acc.z); acc.w = fmaf(v.w, wgt, acc.w);
        }
    }
    s_acc[sg][c4] = acc;
    if (c4 == 0) s_L[sg] = L;
    __syncthreads();
    if (tid < C4) {
        float Lt = 0.f;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int g = 0; g < SG; ++g) {
            const float4 v = s_acc[g][tid];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
            Lt += s_L[g];
        }
        const float inv = (M != -INFINITY) ? 1.f / Lt : 0.f;
        const float r[4] = {t.x * inv, t.y * inv, t.z * inv, t.w * inv};
        if (OUT_BF16) {
            uint16_t h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t u = __float_as_uint(r[e]);
                u += 0x7fffu + ((u >> 16) & 1u); // round to nearest even (finite values)
                h[e] = (uint16_t)(u >> 16);
            }
            uint2 packed = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(o) + row * D + 4 * tid) = packed;
        } else {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(o) + row * D + 4 * tid) = make_float4(r[0], r[1], r[2], r[3]);
        }
        if (tid == 0 && lse) lse[row] = (M != -INFINITY) ? M + logf(Lt) : -INFINITY;
    }
    // log-sum-exp of the first set alone (the window part of a step: its attention weights are normalised by it)
    if (lse_p && tid == kBlock - 1) {
        float Mp = -INFINITY, Lp = 0.f;
        for (int s = 0; s < np; ++s) Mp = fmaxf(Mp, p.m[row * np + s]);
        if (Mp != -INFINITY)
            for (int s = 0; s < np; ++s) Lp = fmaf(p.l[row * np + s], expf(p.m[row * np + s] - Mp), Lp);
        lse_p[row] = (Mp != -INFINITY) ? Mp + logf(Lp) : -INFINITY;
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
                           float *lse, hipStream_t s, float *lse_p)
{
    if (n_rows == 0) return hipSuccess;
    const dim3 grid((unsigned)n_rows), block(kBlock);
    if (head_dim == 64 && o_dtype == 0) HGCA_LAUNCH((combine_kernel<64, false>), grid, block, s, p, q, o, lse, lse_p);
    else if (head_dim == 64 && o_dtype == 1) HGCA_LAUNCH((combine_kernel<64, true>), grid, block, s, p, q, o, lse, lse_p);
    else if (head_dim == 128 && o_dtype == 0) HGCA_LAUNCH((combine_kernel<128, false>), grid, block, s, p, q, o, lse, lse_p);
    else if (head_dim == 128 && o_dtype == 1) HGCA_LAUNCH((combine_kernel<128, true>), grid, block, s, p, q, o, lse, lse_p);
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
