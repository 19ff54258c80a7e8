// Device code shared by the attention kernels: the pieces of one split of softmax attention (scores on the VALU
// or on the matrix cores, softmax statistics of the split, V pass, partial output), written for a workgroup of
// BLOCK threads so that kernels with different workgroup sizes, and kernels that run a split beside other work
// in one launch, use the same code.
#pragma once

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
// bit 0: the gather's first V loads are issued before the split's softmax; bit 1: the window split's as well
#ifndef HGCA_V_PREFETCH
#define HGCA_V_PREFETCH 3
#endif


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

template <int D, int NH, int BLOCK = kBlock>
__device__ __forceinline__ void write_empty_partial(const Partials &part, int64_t bh0, int split)
{
    for (int i = threadIdx.x; i < NH * D; i += BLOCK) {
        const int g = i / D, col = i % D;
        part.o[((bh0 + g) * part.n_splits + split) * D + col] = 0.f;
    }
    if (threadIdx.x < NH) {
        part.m[(bh0 + threadIdx.x) * part.n_splits + split] = -INFINITY;
        part.l[(bh0 + threadIdx.x) * part.n_splits + split] = 0.f;
    }
}

// s_p[g][0..nt) holds scores on entry and weights e^{s-m} on exit; one wave per head.
template <int NH, int BLOCK = kBlock, int LD = kMaxChunk>
__device__ __forceinline__ void split_softmax(float (*s_p)[LD], float *s_m, float *s_l, int nt)
{
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    for (int g = w; g < NH; g += BLOCK / kWave) {
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
// The first UNROLL loads of a lane's V pass (the rows value_pass takes first), for a caller that wants them in
// flight before the weights are ready: the addresses depend on the row map only.
template <typename T, int D, int BLOCK = kBlock, int UNROLL = kUnroll>
__device__ __forceinline__ void value_prefetch(const KernelArgs &a, int nt, const RowMap &rows, uint4 (&vr)[UNROLL])
{
    constexpr int LPR = D / Elem<T>::kPerLoad, RPW = kWave / LPR, RPI = (BLOCK / kWave) * RPW;
    constexpr size_t ROW_BYTES = D * sizeof(T);
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave, r = lane / LPR, c = lane % LPR;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int j = min(u * RPI + w * RPW + r, nt - 1);
        vr[u] = make_uint4(0u, 0u, 0u, 0u);
        if (nt > 0) vr[u] = load16_stream(a.kv.v + rows(j) * ROW_BYTES + c * 16);   // (uniform; a split is never empty here)
    }
}

// V pass of a split: o = sum_j p_j v_j per head, reduced over the workgroup, and the split's partial (m, l, o).
// With PRE the first UNROLL loads of every lane have been issued by value_prefetch (`first`).
template <typename T, int D, int NH, bool GATHER, int BLOCK = kBlock, int UNROLL = kUnroll, int LD = kMaxChunk, bool PRE = false>
__device__ __forceinline__ void value_pass(const KernelArgs &a, float (*s_p)[LD],
                                           float (*s_red)[NH][D], const float *s_m, const float *s_l,
                                           int64_t bh0, int split, int nt, const RowMap &rows,
                                           const uint4 *first = nullptr)
{
    constexpr int EPL = Elem<T>::kPerLoad;       // elements per lane per load
    constexpr int LPR = D / EPL;                 // lanes per row
    constexpr int RPW = kWave / LPR;             // rows per wave per load
    constexpr int NW = BLOCK / kWave;              // waves of the workgroup
    constexpr int RPI = NW * RPW;            // rows per workgroup iteration
    constexpr size_t ROW_BYTES = D * sizeof(T);
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int r = lane / LPR, c = lane % LPR;

    float acc[NH][EPL];
#pragma unroll
    for (int g = 0; g < NH; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    auto consume = [&](int base, const uint4 (&vr)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
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
    };
    if (PRE) {
        uint4 vr[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) vr[u] = first[u];
        consume(0, vr);
    }
    for (int base = PRE ? RPI * UNROLL : 0; base < nt; base += RPI * UNROLL) {
        uint4 vr[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = min(base + u * RPI + w * RPW + r, nt - 1);
            vr[u] = load16_stream(a.kv.v + rows(j) * ROW_BYTES + c * 16);
        }
        consume(base, vr);
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

    for (int i = tid; i < NH * D; i += BLOCK) {
        const int g = i / D, col = i % D;
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) v += s_red[ww][g][col];
        a.part.o[((bh0 + g) * a.part.n_splits + split) * D + col] = v;
    }
    if (tid < NH) {
        a.part.m[(bh0 + tid) * a.part.n_splits + split] = s_m[tid];
        a.part.l[(bh0 + tid) * a.part.n_splits + split] = s_l[tid];
    }
}

// Scaled scores of the split to a.scores[b, h, t0 .. t0+nt) for the NH heads of the workgroup.
template <int NH, int BLOCK = kBlock, int LD = kMaxChunk>
__device__ __forceinline__ void store_split_scores(const KernelArgs &a, const float (*s_p)[LD], int64_t bh0,
                                                   int t0, int nt)
{
    if (a.group_max) {                           // one row per KV head: row index bh0 / NH (bh0 is the group's first head)
        for (int j = threadIdx.x; j < nt; j += BLOCK) {
            float v = s_p[0][j];
#pragma unroll
            for (int g = 1; g < NH; ++g) v = fmaxf(v, s_p[g][j]);
            a.scores[(bh0 / NH) * (int64_t)a.kv.cap + t0 + j] = v;
        }
        return;
    }
    for (int i = threadIdx.x; i < NH * LD; i += BLOCK) {         // indexed by the compile-time row length: no division by nt
        const int g = i / LD, j = i % LD;
        if (j < nt) a.scores[(bh0 + g) * (int64_t)a.kv.cap + t0 + j] = s_p[g][j];
    }
}

// ---- MFMA path (bf16 K/V, dense over a tier) -------------------------------------------------

// One split of softmax attention on the VALU path (any dtype and head_dim): dense over a tier, gathered through a
// list of positions, or the score pass alone.  `unit` is the query head (per-head lists) or the KV head.
// UNROLL: 16-byte loads a lane keeps in flight in the K and V passes.
template <typename T, int D, int NH, int MODE, int UNROLL = kUnroll>
struct SplitValu {
    static constexpr int kPBytes = NH * kMaxChunk * 4, kRowBytes = kMaxChunk * 4, kRedBytes = kWaves * NH * D * 4;
    static constexpr int kLdsBytes = kPBytes + kRowBytes + kRedBytes + 64;

    // lds: kLdsBytes, 16-byte aligned; a workgroup of kBlock threads
    static __device__ __forceinline__ void run(const KernelArgs &a, char *lds, int split, int unit, int b)
    {
        constexpr int EPL = Elem<T>::kPerLoad;
        constexpr int LPR = D / EPL;
        constexpr int RPW = kWave / LPR;
        constexpr int RPI = kWaves * RPW;
        constexpr size_t ROW_BYTES = D * sizeof(T);

        float(*s_p)[kMaxChunk] = reinterpret_cast<float(*)[kMaxChunk]>(lds);          // scores of the split, then weights
        uint32_t *s_row = reinterpret_cast<uint32_t *>(lds + kPBytes);
        float(*s_red)[NH][D] = reinterpret_cast<float(*)[NH][D]>(lds + kPBytes + kRowBytes);
        float *s_m = reinterpret_cast<float *>(lds + kPBytes + kRowBytes + kRedBytes), *s_l = s_m + NH;

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
        for (int base = 0; MODE != kGatherScored && base < nt; base += RPI * UNROLL) {
            uint4 kr[UNROLL];
    #pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int j = min(base + u * RPI + w * RPW + r, nt - 1);
                kr[u] = load16_stream(a.kv.k + rows(j) * ROW_BYTES + c * 16);
            }
    #pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
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

        if (HGCA_V_PREFETCH && GATHER) {             // the first V rows travel while the softmax statistics are formed
            uint4 first[UNROLL];
            value_prefetch<T, D, kBlock, UNROLL>(a, nt, rows, first);
            split_softmax<NH>(s_p, s_m, s_l, nt);
            __syncthreads();
            value_pass<T, D, NH, GATHER, kBlock, UNROLL, kMaxChunk, true>(a, s_p, s_red, s_m, s_l, bh0, split, nt, rows, first);
            return;
        }
        split_softmax<NH>(s_p, s_m, s_l, nt);
        __syncthreads();
        value_pass<T, D, NH, GATHER, kBlock, UNROLL>(a, s_p, s_red, s_m, s_l, bh0, split, nt, rows);
    }
};

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
template <int D, int G, int BLOCK = kBlock, int LD = kMaxChunk>
__device__ __forceinline__ void value_pass_mfma(const KernelArgs &a, float (*s_p)[LD], char *stage,
                                                float (*s_red)[G][D], const float *s_m, const float *s_l, int64_t bh0,
                                                int split, int nt, const RowMap &rows)
{
    constexpr int NW = BLOCK / kWave;
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
    for (int blk = w; blk < n_blocks; blk += NW) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int p = lane + kWave * u, trow = p / PIECES, piece = p % PIECES;
            *reinterpret_cast<uint4 *>(st + trow * VS + 16 * piece) = vr[u];
        }
        if (blk + NW < n_blocks) load_block(blk + NW, vr);
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
    for (int i = tid; i < G * D; i += BLOCK) {
        const int gg = i / D, col = i % D;
        float v = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) v += s_red[ww][gg][col];
        a.part.o[((bh0 + gg) * a.part.n_splits + split) * D + col] = v;
    }
    if (tid < G) {
        a.part.m[(bh0 + tid) * a.part.n_splits + split] = s_m[tid];
        a.part.l[(bh0 + tid) * a.part.n_splits + split] = s_l[tid];
    }
}


// One split of the dense window attention of one (sequence, KV head), by a workgroup of BLOCK threads: scores of
// the split on the matrix cores, softmax statistics of the split in LDS, V pass, one partial (m, l, o) per head.
// A split without tokens (nt == 0) goes through the same barriers and writes the empty partial (m = -inf, l = 0,
// o = 0), so workgroups that run several roles or splits side by side stay in step.
// LD is the largest split the workgroup's LDS is sized for (the caller's chunk must not exceed it).
template <int D, int G, int BLOCK = kBlock, int UNROLL = kUnroll, int LD = kMaxChunk>
struct DenseSplit {
    static constexpr int kNW = BLOCK / kWave;
    // the K stage is dead once the scores are in s_p; the V stage and the output reduction reuse its space
    static constexpr int kStageBytes = kNW * Stage<D>::kWaveVecs * 16;
    static constexpr bool kPvMfma = G >= HGCA_DENSE_PV_MFMA_FROM;
    static constexpr int kVStageBytes = kPvMfma ? kNW * 32 * (D * 2 + kPvPad) : 0;
    static constexpr int kRedBytes = kNW * G * D * 4 + kVStageBytes;
    static constexpr int kBufBytes = kStageBytes > kRedBytes ? kStageBytes : kRedBytes;
    static constexpr int kPBytes = G * LD * 4;
    static constexpr int kStatBytes = 64;                        // s_m[G], s_l[G]
    static constexpr int kLdsBytes = kBufBytes + kPBytes + kStatBytes + LD * 4;

    // lds: kLdsBytes, 16-byte aligned.  t0 .. t0+nt are the split's tokens (nt may be 0).
    static __device__ __forceinline__ void run(const KernelArgs &a, char *lds, int split, int kvh, int b, int t0, int nt)
    {
        char *s_buf = lds;
        float(*s_p)[LD] = reinterpret_cast<float(*)[LD]>(lds + kBufBytes);
        float *s_m = reinterpret_cast<float *>(lds + kBufBytes + kPBytes), *s_l = s_m + G;
        uint32_t *s_row = reinterpret_cast<uint32_t *>(lds + kBufBytes + kPBytes + kStatBytes);
        const int64_t bh0 = (int64_t)b * a.sh.n_q_heads + (int64_t)kvh * G;
        const RowMap rows = make_row_map<false, BLOCK>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0, nt, nullptr);
        mfma_scores<D, G, LD, kNW>(a, reinterpret_cast<uint4 *>(s_buf), s_p, bh0, nt, rows);
        __syncthreads();
        if (a.scores) {                          // uniform over the workgroup
            store_split_scores<G, BLOCK, LD>(a, s_p, bh0, t0, nt);
            __syncthreads();                     // the softmax below overwrites the scores other waves are still storing
        }
        if (HGCA_V_PREFETCH & 2 && !kPvMfma) {       // the first V rows travel while the softmax statistics are formed
            uint4 first[UNROLL];
            value_prefetch<bf16_t, D, BLOCK, UNROLL>(a, nt, rows, first);
            split_softmax<G, BLOCK, LD>(s_p, s_m, s_l, nt);
            __syncthreads();
            value_pass<bf16_t, D, G, false, BLOCK, UNROLL, LD, true>(a, s_p, reinterpret_cast<float(*)[G][D]>(s_buf), s_m,
                                                                     s_l, bh0, split, nt, rows, first);
            return;
        }
        split_softmax<G, BLOCK, LD>(s_p, s_m, s_l, nt);
        __syncthreads();
        if (kPvMfma)                             // V stage first, reduction area behind it
            value_pass_mfma<D, G, BLOCK, LD>(a, s_p, s_buf, reinterpret_cast<float(*)[G][D]>(s_buf + kVStageBytes), s_m, s_l,
                                         bh0, split, nt, rows);
        else
            value_pass<bf16_t, D, G, false, BLOCK, UNROLL, LD>(a, s_p, reinterpret_cast<float(*)[G][D]>(s_buf), s_m, s_l, bh0,
                                                           split, nt, rows);
    }
};

}  // namespace

}  // namespace hgca
