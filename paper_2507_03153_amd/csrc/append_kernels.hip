// Append stage: N queries per sequence attend to one KV tier (Sec. 2.1: S = Q K^T, A = softmax(S),
// O = A V with Q in R^{h x N x d}; Alg. 2, append branch).  bf16 inputs, both contractions on
// v_mfma_f32_16x16x32_bf16.
//
// Work unit of the attention kernel: one workgroup = one split of the tokens of one (sequence, KV head) and up
// to 128 query rows (a row = one query x one head of the GQA group, query-major).  Every wave owns row tiles of 16
// rows, so nothing is reduced across waves.  The K and V rows of a 64-token step are brought into a double-buffered
// LDS stage by LDS-direct loads (no registers in between); the next step's loads are in flight during a step's
// arithmetic, one barrier per step; two workgroups share a CU.  A step is 64 tokens rather than 32 because the
// softmax of a step is one dependent chain (scores, row maximum, exponentials, row sum, rounding, second
// contraction): four score tiles per chain give the wave independent work to overlap it with.
//
// Orientation (per 16-row tile, per step):
//   S^T[token, row]  = K[token, :] . Q[row, :]        A = K tile (LDS, swizzled rows), B = Q (registers)
//   O^T[dcol, row]  += V^T[dcol, token] . P^T[token, row]   A = V^T (LDS transpose reads of the rows), B = P
// In both results a lane's column is the query row lane%16, so the running maximum, the running sum
// and the rescaling factor of a row live in the lanes that hold its scores AND its output columns:
// the online softmax needs two lane exchanges per row statistic and no LDS.  The probabilities go from
// the score registers straight into the B operand of the second contraction (the contraction index
// is matched by reading V^T in the same token order); they are rounded to bf16 there, as a high and a
// low part (two MFMAs, fp32-level accuracy) or, on request, as one part.
//
// The weights kernel brings its K rows in the same way (it has no second contraction).
#include "hgca_launch.hpp"
#include "row_map.hpp"

namespace hgca {

namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));

constexpr int kABlock = 512;
constexpr int kAWaves = kABlock / kWave;
constexpr int kStepBlocks = 2;                   // 32-token contraction blocks per step
constexpr int kStepTokens = 32 * kStepBlocks;
constexpr int kRowsPerBlock = 128;               // query rows per workgroup = 8 tiles of 16, one per wave
static_assert(kRowsPerBlock == 16 * kAWaves, "one row tile per wave");
constexpr int kSub = kMaxChunk;                  // entries of the table of block rows (paged tiers)

// Where the rows of a pass over part of a split live.  A contiguous tier is plain arithmetic.  A paged tier gets a
// table in LDS with one entry per BLOCK the pass touches (the row of the block's first token for this KV head), so
// one filling of kSub entries covers (kSub - 1) * block_size tokens -- a whole split for blocks of 16 tokens -- and
// the load pipeline is not drained for refills.
struct BlockRows {
    const uint32_t *table;                       // LDS; nullptr => row = base + j
    uint32_t base;
    int32_t bs, shift, off;                      // block size, log2 of it (-1: not a power of two), first token's place in its block
    __device__ __forceinline__ uint32_t operator()(int j) const {
        if (!table) return base + (uint32_t)j;
        const int t = off + j;
        return shift >= 0 ? table[t >> shift] + (uint32_t)(t & (bs - 1)) : table[t / bs] + (uint32_t)(t % bs);
    }
};

// tokens a pass may cover so that its blocks fit the table, a multiple of the step
__device__ __forceinline__ int pass_length(const KvDev &kv, int nt_total) {
    if (!kv.block_table) return max(nt_total, 1);
    const int64_t t = (int64_t)(kSub - 1) * kv.block_size;
    return (int)max((int64_t)kStepTokens, min(t, (int64_t)1 << 30) / kStepTokens * kStepTokens);
}

// `first` is the tier position of the pass's first token, nt the number of tokens; contains a barrier iff the tier
// is paged (uniform over the workgroup).
template <int BLOCK>
__device__ __forceinline__ BlockRows make_block_rows(uint32_t *s_tab, const KvDev &kv, int n_kv_heads, int b, int kvh,
                                                     int first, int nt)
{
    b = kv_seq(kv, b);
    BlockRows m;
    m.bs = max(kv.block_size, 1);
    m.shift = (m.bs & (m.bs - 1)) == 0 ? __builtin_ctz(m.bs) : -1;
    if (!kv.block_table) {
        m.table = nullptr;
        m.base = (uint32_t)(((int64_t)b * n_kv_heads + kvh) * kv.cap + first);
        m.off = 0;
        return m;
    }
    const int32_t *blocks = kv.block_table + (int64_t)b * kv.max_blocks + (kv.first_block ? kv.first_block[b] : 0);
    const int blk0 = first / m.bs, n_blk = (first + nt - 1) / m.bs - blk0 + 1;      // <= kSub by pass_length
    for (int i = threadIdx.x; i < n_blk; i += BLOCK)
        s_tab[i] = (uint32_t)(((int64_t)blocks[blk0 + i] * n_kv_heads + kvh) * m.bs);
    __syncthreads();
    m.table = s_tab;
    m.base = 0;
    m.off = first - blk0 * m.bs;
    return m;
}

// The value of the lane ROT places further on in the same row of 16 lanes (DPP row_ror).
template <int ROT>
__device__ __forceinline__ float row_rotate(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + ROT, 0xf, 0xf, true));
}

// Reductions over the four 16-lane rows of a wave (lanes n, n + 16, n + 32, n + 48 hold partial results of one
// query row).  v_permlane16_swap / v_permlane32_swap of a register with itself return (rows 0 0 2 2, rows 1 1 3 3)
// and (lower half twice, upper half twice): two VALU instructions per level where a lane shuffle would go through
// the LDS pipeline, which matters because the row maximum heads the dependent chain of every step.
__device__ __forceinline__ float rows_max(float x) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
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

// Raw scores <q, k> (no softmax scale yet) of one 16-row tile for the step's tokens: sv[8*kb + 4*tt + r] belongs
// to step token 32*kb + 16*tt + 4*g + r and query row lane % 16.  With MASK, tokens at or beyond `limit` (counted
// from the step's first token) read -inf.
// `k_piece(t, kk)` reads this lane's A operand: 8 elements from column 32 kk + 8 (lane / 16) on of the K row of
// token 16 t + lane % 16 of the step.
template <int D, bool MASK, typename KPiece>
__device__ __forceinline__ void tile_scores(KPiece k_piece, const bf16x8 (&qop)[D / 32], int limit,
                                            float (&sv)[8 * kStepBlocks])
{
    const int lane = threadIdx.x % kWave, g = lane / 16;
#pragma unroll
    for (int t = 0; t < 2 * kStepBlocks; ++t) {  // 16-token tiles of the step
        floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            const uint4 ka = k_piece(t, kk);
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qop[kk], c, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sv[4 * t + r] = (!MASK || 16 * t + 4 * g + r < limit) ? c[r] : -INFINITY;
    }
}

#ifndef HGCA_APPEND_PV_GROUP
#define HGCA_APPEND_PV_GROUP 4
#endif
#ifndef HGCA_APPEND_TILES
#define HGCA_APPEND_TILES 2
#endif

// LDS stage of the attention kernel: the rows of a step are brought in by LDS-direct loads (global_load_lds, 16
// bytes per lane, no registers in between).  One such instruction fills 1024 consecutive bytes of LDS with whatever
// 64 pieces its lanes address, so the layout inside each 1 KB group is chosen by the lane -> global address map:
//   K: row-major rows with the 16-byte pieces of a row XOR-swizzled by the row, so that the 16 rows an A-operand
//      read touches land on different banks without padding;
//   V: the group's rows interleaved in 32-byte chunks ([column chunk][row][32 bytes]), so that the 4 rows x 32 bytes
//      a 16-lane group takes with one transpose read are 128 consecutive bytes.
template <int D, int NW> struct DmaStage {
    static constexpr int kPieces = D / 8;                        // 16-byte pieces per row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kGroupRows = 1024 / kRowBytes;          // rows per load instruction of a wave
    static constexpr int kGroups = kStepTokens / kGroupRows;     // per step and tensor
    static constexpr int kLoads = kGroups / NW;                  // per wave, step and tensor
    static constexpr int kBytes = kStepTokens * kRowBytes;       // per step and tensor
    static_assert(kGroups % NW == 0 && kLoads >= 1, "the waves share the groups of a step evenly");

    static __device__ __forceinline__ int k_swizzle(int row) { return (row / (16 / kPieces)) % kPieces; }
    // byte offset, in a K stage, of logical piece `piece` of step row `row`
    static __device__ __forceinline__ int k_offset(int row, int piece) {
        return row * kRowBytes + 16 * (piece ^ k_swizzle(row));
    }
    // byte offset, in a V stage, of the 32-byte column chunk `dt` of step row `row`
    static __device__ __forceinline__ int v_offset(int row, int dt) {
        return (row / kGroupRows) * 1024 + dt * (kGroupRows * 32) + (row % kGroupRows) * 32;
    }
};

// s_waitcnt vmcnt(0) (expcnt and lgkmcnt fields at their maxima = no wait): an LDS-direct load has landed in LDS
// when the wave's memory-load counter has counted it down.  Every wave does this before the barrier after which
// other waves read what it loaded.
__device__ __forceinline__ void wait_for_own_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Requests the K and the V rows of a step.  All row numbers are looked up before the first load is issued: the
// lookup of a paged tier reads a table in LDS, and an LDS read placed after an LDS-direct load waits for that load.
template <int D, int NW, bool WITH_V = true>
__device__ __forceinline__ void dma_step(const KvDev &kv, const BlockRows &rows, int step, int nsub, char *k_stage,
                                         char *v_stage)
{
    using S = DmaStage<D, NW>;
    const int lane = threadIdx.x % kWave, w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const char *k_src[S::kLoads], *v_src[S::kLoads];
#pragma unroll
    for (int u = 0; u < S::kLoads; ++u) {
        const int group = w + NW * u;                            // uniform over the wave
        // what lands at byte 16 * lane of the group: K row-major with swizzled pieces, V chunk-interleaved
        const int k_row = group * S::kGroupRows + lane / S::kPieces;
        const int k_piece = (lane % S::kPieces) ^ S::k_swizzle(k_row);
        const int v_row = group * S::kGroupRows + (lane / 2) % S::kGroupRows;
        const int v_piece = 2 * (lane / (2 * S::kGroupRows)) + lane % 2;
        k_src[u] = kv.k + (size_t)rows(min(step * kStepTokens + k_row, nsub - 1)) * S::kRowBytes + 16 * k_piece;
        if (WITH_V) v_src[u] = kv.v + (size_t)rows(min(step * kStepTokens + v_row, nsub - 1)) * S::kRowBytes + 16 * v_piece;
    }
#pragma unroll
    for (int u = 0; u < S::kLoads; ++u) {
        const int group = w + NW * u;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)k_src[u],
                                         (__attribute__((address_space(3))) void *)(k_stage + group * 1024), 16, 0, 0);
        if (WITH_V)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)v_src[u],
                                             (__attribute__((address_space(3))) void *)(v_stage + group * 1024), 16, 0, 0);
    }
}

// TILES row tiles of 16 query rows per wave (128 rows per workgroup, so 8 / TILES waves): with two tiles every K
// and V operand read from LDS feeds two matrix instructions, and the two tiles' softmax chains are independent
// work for the wave to overlap.
//
// A launch may serve TWO tiers (the window and the complete pool of an append turn: Alg. 2 runs the two attentions
// side by side): the first a1.part.n_splits workgroups along x take the splits of a1, the rest those of a2, each
// with its tier's view, mask rule, split size and partials; everything else (queries, shape) is common.  One launch
// then pays one ramp-up and one tail, and the short tier's splits can be as long as the long tier's.
template <int D, int G, bool SPLIT_P, int TILES>
__global__ __launch_bounds__(kABlock / TILES, 4 / TILES) void append_attn_kernel(AppendArgs a1, AppendArgs a2)
{
    const bool second = (int)blockIdx.x >= a1.part.n_splits;     // uniform over the workgroup
    const AppendArgs &a = second ? a2 : a1;
    constexpr int NW = kAWaves / TILES, BLOCK = NW * kWave;
    using S = DmaStage<D, NW>;
    constexpr int DT = D / 16;
    constexpr float kLog2e = 1.4426950408889634f;
    // two stages per tensor as separate arrays: the compiler then knows that a load into one stage does not
    // touch the other and lets the reads of the current stage go ahead while the next one is being filled
    __shared__ __attribute__((aligned(1024))) char s_k0[S::kBytes];
    __shared__ __attribute__((aligned(1024))) char s_k1[S::kBytes];
    __shared__ __attribute__((aligned(1024))) char s_v0[S::kBytes];
    __shared__ __attribute__((aligned(1024))) char s_v1[S::kBytes];
    __shared__ uint32_t s_row[kSub];

    const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
    const int split = (int)blockIdx.x - (second ? a1.part.n_splits : 0);
    const int kvh = blockIdx.y / n_qb, qb = blockIdx.y % n_qb, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    // the tier's actual length is shared out evenly among its splits (a.chunk, set from the capacity, bounds it):
    // every split of a sequence then has the same work however far its length is from the capacity
    const int chunk = min(a.chunk, ((len + a.part.n_splits - 1) / a.part.n_splits + kStepTokens - 1) / kStepTokens * kStepTokens);
    const int t0 = split * chunk;
    const int nt_total = min(chunk, len - t0);                   // <= 0: nothing of this split is valid

    const int tile_row0 = qb * kRowsPerBlock + w * 16 * TILES;   // first row of the wave's first tile
    const bool wave_live = tile_row0 < a.n_q * G;                // uniform over the wave
    RowInfo ri[TILES];
    int vis[TILES];                              // tokens [0, vis) of the tier are visible to the row
    int vis_min = INT32_MAX;                     // over the rows of the wave: steps below it need no mask
    bf16x8 qop[TILES][D / 32];
#pragma unroll
    for (int x = 0; x < TILES; ++x) {
        ri[x] = row_info<G>(a, b, kvh, tile_row0 + 16 * x + n);
        vis[x] = !ri[x].valid ? 0 : a.causal_tail ? min(max(len - a.n_q + ri[x].query + 1, 0), len) : len;
        vis_min = min(vis_min, vis[x]);
        load_q_tile<D>(a, ri[x], g, qop[x]);
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) vis_min = min(vis_min, __shfl_xor(vis_min, off, kWave));
    // The running maximum m is kept on the RAW scores (the softmax scale is positive, so the order is the same) and
    // the scale, in units of ln 2, is applied inside the exponent: e^{scale (s - m)} = 2^{fma(s, scale2, -m scale2)},
    // one fused multiply-add and one bare v_exp_f32 per score.
    const float scale2 = a.sh.sm_scale * kLog2e;
    float m[TILES], l[TILES];
    floatx4 acc[TILES][DT];
#pragma unroll
    for (int x = 0; x < TILES; ++x) {
        m[x] = -INFINITY;
        l[x] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc[x][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // this lane's byte offsets into a stage: the A operand of the first product (row n of a 16-token tile, one
    // offset per 32-column slice because of the swizzle) and of the second.  The V^T operand (8 tokens of one column
    // per lane) comes from two transpose reads: lane j of a group points at columns 4(j%4).. of the row of
    // contraction index j/4 (first read) and 4 + j/4 (second read).
    int k_lane[D / 32];
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) k_lane[kk] = S::k_offset(n, 4 * kk + g);
    const int v_lane_lo = S::v_offset(block_token(g, n / 4), 0) + 8 * (n % 4);
    const int v_lane_hi = S::v_offset(block_token(g, 4 + n / 4), 0) + 8 * (n % 4);

    auto step_body = [&](const char *k_stage, const char *v_stage, int step0, int in_split) {
        // raw scores: sv[x][8*kb + 4*tt + r] belongs to step token 32*kb + 16*tt + 4*g + r and row n of tile x
        float sv[TILES][8 * kStepBlocks];
        const bool masked = min(in_split, vis_min - step0) < kStepTokens;   // uniform over the wave
        {
            // the slices of the contraction outermost: the 4 x TILES accumulators take turns, so no matrix instruction
            // waits for the one before it on the same accumulator
            constexpr int NT = 2 * kStepBlocks;                  // 16-token tiles of the step
            floatx4 c[NT][TILES];
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int x = 0; x < TILES; ++x) c[t][x] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint4 ka = *reinterpret_cast<const uint4 *>(k_stage + t * 16 * S::kRowBytes + k_lane[kk]);
#pragma unroll
                    for (int x = 0; x < TILES; ++x)
                        c[t][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qop[x][kk], c[t][x], 0, 0, 0);
                }
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int x = 0; x < TILES; ++x)
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[x][4 * t + r] = c[t][x][r];
        }
        if (masked) {                                            // steps that touch a length or causal boundary
            asm volatile("" ::: "memory");                       // a real branch: the selects below are not speculated into every step
#pragma unroll
            for (int x = 0; x < TILES; ++x) {
                const int limit = min(in_split, vis[x] - step0);
#pragma unroll
                for (int e = 0; e < 8 * kStepBlocks; ++e)
                    if (16 * (e / 4) + 4 * g + e % 4 >= limit) sv[x][e] = -INFINITY;
            }
        }
        bf16x8 ph[TILES][kStepBlocks], pl[TILES][kStepBlocks];
#pragma unroll
        for (int x = 0; x < TILES; ++x) {
            float mx = sv[x][0];
#pragma unroll
            for (int e = 1; e < 8 * kStepBlocks; ++e) mx = fmaxf(mx, sv[x][e]);
            const float m_new = fmaxf(m[x], rows_max(mx));
            // a row that has seen nothing yet keeps m = -inf: shift by 0 then, every exponent is -inf and gives 0
            const float shift = (m_new == -INFINITY) ? 0.f : -m_new * scale2;
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8 * kStepBlocks; ++e) {          // sv becomes the probabilities; masked scores give 0
                sv[x][e] = __builtin_amdgcn_exp2f(fmaf(sv[x][e], scale2, shift));
                ps += sv[x][e];
            }
            const float corr = (m[x] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(fmaf(m[x], scale2, shift));
            l[x] = l[x] * corr + rows_sum(ps);
            m[x] = m_new;
            if (__any(corr != 1.f)) {                            // once the maxima have settled nothing is rescaled
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc[x][dt] *= corr;
            }
            // round to nearest even, two weights per conversion; the low part carries the rounding error: the high
            // parts are widened again from the packed pair (a shift and a mask) rather than converted one by one
#pragma unroll
            for (int kb = 0; kb < kStepBlocks; ++kb) {
                uint32_t hw[4], lw[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float2v pr = {sv[x][8 * kb + 2 * e2], sv[x][8 * kb + 2 * e2 + 1]};
                    hw[e2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                    lw[e2] = 0u;
                    if (SPLIT_P) {
                        const float2v lo = {pr[0] - __uint_as_float(hw[e2] << 16), pr[1] - __uint_as_float(hw[e2] & 0xffff0000u)};
                        lw[e2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
                    }
                }
                ph[x][kb] = __builtin_bit_cast(bf16x8, make_uint4(hw[0], hw[1], hw[2], hw[3]));
                pl[x][kb] = __builtin_bit_cast(bf16x8, make_uint4(lw[0], lw[1], lw[2], lw[3]));
            }
        }
        // O^T += V^T P^T, one 16-column tile of the output at a time
#pragma unroll
        for (int kb = 0; kb < kStepBlocks; ++kb) {
            const char *v_lo = v_stage + S::v_offset(32 * kb, 0) + v_lane_lo;
            const char *v_hi = v_stage + S::v_offset(32 * kb, 0) + v_lane_hi;
            // column tiles in groups of kPvGroup: the group's high-part products first, then its low-part ones, so
            // that two MFMAs on the same accumulator are several instructions apart
            constexpr int kPvGroup = HGCA_APPEND_PV_GROUP;
#pragma unroll
            for (int dt0 = 0; dt0 < DT; dt0 += kPvGroup) {
                bf16x8 vop[kPvGroup];
#pragma unroll
                for (int u = 0; u < kPvGroup; ++u) {
                    const int at = S::v_offset(0, dt0 + u);
                    const short4v a0 = lds_read_tr16(v_lo + at), a1 = lds_read_tr16(v_hi + at);
                    const short8v both = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                    vop[u] = __builtin_bit_cast(bf16x8, both);
                }
#pragma unroll
                for (int x = 0; x < TILES; ++x)
#pragma unroll
                    for (int u = 0; u < kPvGroup; ++u)
                        acc[x][dt0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[u], ph[x][kb], acc[x][dt0 + u], 0, 0, 0);
                if (SPLIT_P) {
#pragma unroll
                    for (int x = 0; x < TILES; ++x)
#pragma unroll
                        for (int u = 0; u < kPvGroup; ++u)
                            acc[x][dt0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[u], pl[x][kb], acc[x][dt0 + u], 0, 0, 0);
                }
            }
        }
    };

    // a paged tier needs a table of block rows in LDS, which covers a whole split unless the blocks are tiny;
    // a contiguous tier is plain arithmetic
    const int sub_len = pass_length(a.kv, nt_total);
    for (int sub0 = 0; sub0 < nt_total; sub0 += sub_len) {
        const int nsub = min(sub_len, nt_total - sub0);
        __syncthreads();                         // the previous table and stages are no longer in use
        const BlockRows rows = make_block_rows<BLOCK>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0 + sub0, nsub);
        // Step s reads the stages of its parity and requests the rows of step s + 1 into the stages of the other
        // parity, which were last read in step s - 1: the barrier at the top of the step (before which every wave
        // waits for its own loads) orders both.
        const int steps = (nsub + kStepTokens - 1) / kStepTokens;
        dma_step<D, NW>(a.kv, rows, 0, nsub, s_k0, s_v0);
        auto step = [&](int s, const char *k_cur, const char *v_cur, char *k_next, char *v_next) {
            wait_for_own_loads();                // the barrier alone does not wait for LDS-direct loads
            __syncthreads();
            if (s + 1 < steps) dma_step<D, NW>(a.kv, rows, s + 1, nsub, k_next, v_next);
            if (wave_live) step_body(k_cur, v_cur, t0 + sub0 + s * kStepTokens, nsub - s * kStepTokens);
        };
        for (int s2 = 0; s2 < steps; s2 += 2) {
            step(s2, s_k0, s_v0, s_k1, s_v1);
            if (s2 + 1 < steps) step(s2 + 1, s_k1, s_v1, s_k0, s_v0);
        }
    }

    // partial of every valid row: lane (n, g) holds output columns dt*16 + 4g .. +3 of row n of each tile
#pragma unroll
    for (int x = 0; x < TILES; ++x) {
        if (!ri[x].valid) continue;
        const int64_t at = ri[x].out_row * a.part.n_splits + split;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            *reinterpret_cast<float4 *>(a.part.o + at * D + dt * 16 + 4 * g) =
                make_float4(acc[x][dt][0], acc[x][dt][1], acc[x][dt][2], acc[x][dt][3]);
        if (g == 0) {
            a.part.m[at] = m[x] * a.sh.sm_scale; // the maximum of the scaled scores (-inf stays -inf)
            a.part.l[at] = l[x];
        }
    }
}

// Query-averaged softmax weights of a tier: a_out[b, h, t] = (1/N) sum_i e^{s_it - lse_i} over the queries i
// that see token t (lse_i is the tier's own log-sum-exp for query i), 0 beyond the length.  One workgroup
// owns a_out[b, heads of kvh, t0 .. t0 + chunk): every step the waves' sums go through LDS to one thread
// per entry, which writes (first block of 128 query rows) or adds to (further blocks) the entry.
template <int D, int G>
__global__ __launch_bounds__(kABlock) void append_weights_kernel(AppendArgs a1, AppendArgs a2, int n1)
{
    // a launch may serve two tiers: the first n1 workgroups along x take chunks of a1's tier, the rest of a2's
    const bool second = (int)blockIdx.x >= n1;                   // uniform over the workgroup
    const AppendArgs &a = second ? a2 : a1;
    using S = DmaStage<D, kAWaves>;
    // the K rows of a step arrive by LDS-direct loads, as in the attention kernel: two stages as separate arrays
    __shared__ __attribute__((aligned(1024))) char s_k0[S::kBytes];
    __shared__ __attribute__((aligned(1024))) char s_k1[S::kBytes];
    __shared__ uint32_t s_row[kSub];
    __shared__ __attribute__((aligned(16))) float s_part[2][kAWaves][G][kStepTokens];   // read after the next step's barrier

    const int chunk_id = (int)blockIdx.x - (second ? n1 : 0), kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave, n = lane % 16, g = lane / 16;
    const int len = tier_len(a.kv, b);
    const int t0 = chunk_id * a.chunk;
    const int n_here = min(a.chunk, a.kv.cap - t0);              // entries of a_out this workgroup writes
    const int nt_total = min(a.chunk, len - t0);                 // valid tokens among them (may be <= 0)
    const float inv_n = 1.f / (float)a.n_q;
    constexpr float kLog2e = 1.4426950408889634f;
    const float scale2 = a.sh.sm_scale * kLog2e;
    float *out = a.a_out + ((int64_t)b * a.sh.n_q_heads + kvh * G) * a.kv.cap + t0;

    int k_lane[D / 32];                          // this lane's A-operand offsets in a stage (swizzled pieces)
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) k_lane[kk] = S::k_offset(n, 4 * kk + g);

    const int n_qb = (a.n_q * G + kRowsPerBlock - 1) / kRowsPerBlock;
    const int sub_len = pass_length(a.kv, nt_total);
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
            const BlockRows rows = make_block_rows<kABlock>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0 + sub0, nsub);
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
            // Step s reads the stage of its parity and requests the rows of step s + 1 into the other one, which was
            // last read in step s - 1; the sums of step s - 1 wait in s_part and are folded after the same barrier.
            const int steps = (nsub + kStepTokens - 1) / kStepTokens;
            dma_step<D, kAWaves, false>(a.kv, rows, 0, nsub, s_k0, nullptr);
            auto step = [&](int s, const char *k_cur, char *k_next) {
                wait_for_own_loads();            // the barrier alone does not wait for LDS-direct loads
                __syncthreads();
                if (pending >= 0) fold(pending);                 // written before the barrier above
                if (s + 1 < steps) dma_step<D, kAWaves, false>(a.kv, rows, s + 1, nsub, k_next, nullptr);
                float sv[8 * kStepBlocks];
                const int step0 = sub0 + s * kStepTokens;
                tile_scores<D, true>(
                    [&](int t, int kk) {
                        return *reinterpret_cast<const uint4 *>(k_cur + t * 16 * S::kRowBytes + k_lane[kk]);
                    },
                    qop, min(nsub - s * kStepTokens, vis - (t0 + step0)), sv);
#pragma unroll
                for (int e = 0; e < 8 * kStepBlocks; ++e) {
                    float x = __builtin_amdgcn_exp2f(fmaf(sv[e], scale2, neg_lse2));
                    // add the rows of the same head: columns n, n + G, n + 2G, ... of the 16-lane row, by rotating
                    // the row (DPP row_ror) by 8, 4, ... G lanes
                    if (G <= 8) x += row_rotate<8>(x);
                    if (G <= 4) x += row_rotate<4>(x);
                    if (G <= 2) x += row_rotate<2>(x);
                    if (G <= 1) x += row_rotate<1>(x);
                    sv[e] = x;
                }
                if (n < G) {                     // tokens 16 t + 4 g .. + 3 of the step, head n of the group
#pragma unroll
                    for (int t = 0; t < 2 * kStepBlocks; ++t)
                        *reinterpret_cast<float4 *>(&s_part[s & 1][w][n][16 * t + 4 * g]) =
                            make_float4(sv[4 * t], sv[4 * t + 1], sv[4 * t + 2], sv[4 * t + 3]);
                }
                pending = s;
            };
            for (int s2 = 0; s2 < steps; s2 += 2) {
                step(s2, s_k0, s_k1);
                if (s2 + 1 < steps) step(s2 + 1, s_k1, s_k0);
            }
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

// The same weights for fp32 inputs, on the VALU (the fp32 shapes are the small, exact ones: this pass is written for
// clarity, not for bandwidth).  One workgroup = 64 tokens of one (sequence, KV head): their K rows are parked in LDS
// (one pad per row, a thread walks its own row); thread (t, part) adds e^{s_it - lse_i} over the queries
// i = part, part + 4, ... for every head of the group, the four parts are added through LDS.
constexpr int kF32Tokens = 64, kF32Block = 256, kF32Parts = kF32Block / kF32Tokens;

template <int D, int G>
__global__ __launch_bounds__(kF32Block) void append_weights_f32_kernel(AppendArgs a)
{
    __shared__ float s_k[kF32Tokens][D + 1];
    __shared__ float s_q[kF32Parts][D];
    __shared__ float s_sum[kF32Parts][G][kF32Tokens];
    __shared__ uint32_t s_row[kF32Tokens];

    const int chunk_id = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, t = tid % kF32Tokens, part = tid / kF32Tokens;
    const int len = tier_len(a.kv, b);
    const int t0 = chunk_id * kF32Tokens;
    const int n_here = min(kF32Tokens, a.kv.cap - t0);           // entries of a_out this workgroup writes
    const int nt = min(kF32Tokens, len - t0);                    // valid tokens among them (may be <= 0)
    float *out = a.a_out + ((int64_t)b * a.sh.n_q_heads + kvh * G) * a.kv.cap + t0;
    if (nt <= 0) {                                               // uniform over the workgroup
        for (int i = tid; i < G * n_here; i += kF32Block) out[(int64_t)(i / n_here) * a.kv.cap + i % n_here] = 0.f;
        return;
    }
    const RowMap rows = make_row_map<false, kF32Block>(s_row, a.kv, a.sh.n_kv_heads, b, kvh, t0, nt, nullptr);
    const float *k = reinterpret_cast<const float *>(a.kv.k);
    for (int i = tid; i < nt * D; i += kF32Block) s_k[i / D][i % D] = k[(int64_t)rows(i / D) * D + i % D];
    const float *q = static_cast<const float *>(a.q);
    float acc[G];
#pragma unroll
    for (int gh = 0; gh < G; ++gh) acc[gh] = 0.f;
    const int rounds = (a.n_q + kF32Parts - 1) / kF32Parts;
    for (int gh = 0; gh < G; ++gh) {
        const int h = kvh * G + gh;
        for (int r = 0; r < rounds; ++r) {
            const int i = r * kF32Parts + part;                  // this part's query of the round
            __syncthreads();                                     // the K rows are in place; the previous query is done with
            if (i < a.n_q)
                for (int e = t; e < D; e += kF32Tokens) s_q[part][e] = q[(((int64_t)b * a.n_q + i) * a.sh.n_q_heads + h) * D + e];
            __syncthreads();
            if (i >= a.n_q || t >= nt) continue;                 // no barrier below this line inside the round
            const int vis = a.causal_tail ? min(max(len - a.n_q + i + 1, 0), len) : len;
            if (t0 + t >= vis) continue;
            float dot = 0.f;
#pragma unroll 8
            for (int e = 0; e < D; ++e) dot = fmaf(s_q[part][e], s_k[t][e], dot);
            acc[gh] += expf(dot * a.sh.sm_scale - a.lse[((int64_t)b * a.n_q + i) * a.sh.n_q_heads + h]);
        }
    }
#pragma unroll
    for (int gh = 0; gh < G; ++gh) s_sum[part][gh][t] = acc[gh];
    __syncthreads();
    const float inv_n = 1.f / (float)a.n_q;
    for (int i = tid; i < G * n_here; i += kF32Block) {
        const int gh = i / n_here, j = i % n_here;
        float v = 0.f;
#pragma unroll
        for (int p = 0; p < kF32Parts; ++p) v += s_sum[p][gh][j];
        out[(int64_t)gh * a.kv.cap + j] = j < nt ? v * inv_n : 0.f;
    }
}

template <int D>
hipError_t launch_weights_f32_group(const AppendArgs &a, dim3 grid, hipStream_t s)
{
    switch (a.sh.group) {
    case 1: hipLaunchKernelGGL((append_weights_f32_kernel<D, 1>), grid, dim3(kF32Block), 0, s, a); break;
    case 2: hipLaunchKernelGGL((append_weights_f32_kernel<D, 2>), grid, dim3(kF32Block), 0, s, a); break;
    case 4: hipLaunchKernelGGL((append_weights_f32_kernel<D, 4>), grid, dim3(kF32Block), 0, s, a); break;
    case 8: hipLaunchKernelGGL((append_weights_f32_kernel<D, 8>), grid, dim3(kF32Block), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D, bool SPLIT_P>
hipError_t launch_attn_group(const AppendArgs &a, const AppendArgs &a2, dim3 grid, hipStream_t s)
{
    constexpr int T = HGCA_APPEND_TILES;
    const dim3 block(kABlock / T);
    switch (a.sh.group) {
    case 1: hipLaunchKernelGGL((append_attn_kernel<D, 1, SPLIT_P, T>), grid, block, 0, s, a, a2); break;
    case 2: hipLaunchKernelGGL((append_attn_kernel<D, 2, SPLIT_P, T>), grid, block, 0, s, a, a2); break;
    case 4: hipLaunchKernelGGL((append_attn_kernel<D, 4, SPLIT_P, T>), grid, block, 0, s, a, a2); break;
    case 8: hipLaunchKernelGGL((append_attn_kernel<D, 8, SPLIT_P, T>), grid, block, 0, s, a, a2); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D>
hipError_t launch_weights_group(const AppendArgs &a, const AppendArgs &a2, int n1, dim3 grid, hipStream_t s)
{
    switch (a.sh.group) {
    case 1: hipLaunchKernelGGL((append_weights_kernel<D, 1>), grid, dim3(kABlock), 0, s, a, a2, n1); break;
    case 2: hipLaunchKernelGGL((append_weights_kernel<D, 2>), grid, dim3(kABlock), 0, s, a, a2, n1); break;
    case 4: hipLaunchKernelGGL((append_weights_kernel<D, 4>), grid, dim3(kABlock), 0, s, a, a2, n1); break;
    case 8: hipLaunchKernelGGL((append_weights_kernel<D, 8>), grid, dim3(kABlock), 0, s, a, a2, n1); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_append_attn2(int head_dim, const AppendArgs &a, const AppendArgs &a2, hipStream_t s)
{
    const int n_splits = a.part.n_splits + a2.part.n_splits;
    if (a.sh.batch == 0 || a.n_q == 0 || n_splits == 0) return hipSuccess;
    if (a2.part.n_splits > 0 && (a2.n_q != a.n_q || a2.one_part_p != a.one_part_p || a2.q != a.q || a2.sh.group != a.sh.group ||
                                 a2.sh.batch != a.sh.batch || a2.sh.n_kv_heads != a.sh.n_kv_heads))
        return hipErrorInvalidValue;             // the two tiers share the queries and the launch shape
    const int n_qb = (a.n_q * a.sh.group + kRowsPerBlock - 1) / kRowsPerBlock;
    dim3 grid(n_splits, a.sh.n_kv_heads * n_qb, a.sh.batch);
    if (head_dim == 64)
        return a.one_part_p ? launch_attn_group<64, false>(a, a2, grid, s) : launch_attn_group<64, true>(a, a2, grid, s);
    if (head_dim == 128)
        return a.one_part_p ? launch_attn_group<128, false>(a, a2, grid, s) : launch_attn_group<128, true>(a, a2, grid, s);
    return hipErrorInvalidValue;
}

hipError_t launch_append_attn(int head_dim, const AppendArgs &a, hipStream_t s)
{
    AppendArgs none = a;                         // no second tier: every workgroup takes a split of `a`
    none.part.n_splits = 0;
    return launch_append_attn2(head_dim, a, none, s);
}

hipError_t launch_append_weights2(int head_dim, const AppendArgs &a, int n_chunks, const AppendArgs &a2, int n_chunks2,
                                  hipStream_t s)
{
    if (a.sh.batch == 0 || n_chunks + n_chunks2 == 0) return hipSuccess;
    if (n_chunks2 > 0 && (a2.n_q != a.n_q || a2.q != a.q || a2.sh.group != a.sh.group || a2.sh.batch != a.sh.batch ||
                          a2.sh.n_kv_heads != a.sh.n_kv_heads))
        return hipErrorInvalidValue;             // the two tiers share the queries and the launch shape
    dim3 grid(n_chunks + n_chunks2, a.sh.n_kv_heads, a.sh.batch);
    if (head_dim == 64) return launch_weights_group<64>(a, a2, n_chunks, grid, s);
    if (head_dim == 128) return launch_weights_group<128>(a, a2, n_chunks, grid, s);
    return hipErrorInvalidValue;
}

hipError_t launch_append_weights(int head_dim, const AppendArgs &a, int n_chunks, hipStream_t s)
{
    return launch_append_weights2(head_dim, a, n_chunks, a, 0, s);
}

hipError_t launch_append_weights_f32(int head_dim, const AppendArgs &a, hipStream_t s)
{
    if (a.sh.batch == 0 || a.kv.cap == 0) return hipSuccess;
    dim3 grid((a.kv.cap + kF32Tokens - 1) / kF32Tokens, a.sh.n_kv_heads, a.sh.batch);
    if (head_dim == 64) return launch_weights_f32_group<64>(a, grid, s);
    if (head_dim == 128) return launch_weights_f32_group<128>(a, grid, s);
    return hipErrorInvalidValue;
}

}  // namespace hgca
