// Independent kernels of a decode step as ONE launch.
#include "attn_device.hpp"

namespace hgca {

namespace {

// The window's split kernels and the sparse part's split kernels:
//
// Both are streaming passes that need nothing from each other (Alg. 2 runs gpu_attention and cpu_attention side by
// side); as two launches of one stream the second waits for the last workgroup of the first, and each pays its own
// ramp-up and tail.  In one grid the workgroups of the sparse part take over compute units as the window's
// workgroups drain (or the other way round).  Roles by blockIdx; measured on the 8B shape: with K and V gathered
// (270 MB against the window's 134 MB) the gather's workgroups go first (68.0 against 69.2 us per step), with V
// alone gathered (135 MB) the window's (145.8 against 148.3 us per step with a selection).
#ifndef HGCA_DG_OCC
#define HGCA_DG_OCC 5                            // waves per SIMD the register budget is set for
#endif
#ifndef HGCA_DG_GATHER_UNROLL
#define HGCA_DG_GATHER_UNROLL 8                  // K / V loads a lane of a sparse split keeps in flight (4 in a launch of
#endif                                           // its own, where eight 64-register workgroups share a unit; here the
                                                 // register budget is the window body's: 66.8 against 67.9 us per steady step)
#ifndef HGCA_DG_UNROLL
#define HGCA_DG_UNROLL 4                         // V loads a lane of a window split keeps in flight
#endif

template <int D, int G, int GMODE, int LD>
__global__ __launch_bounds__(kBlock, HGCA_DG_OCC) void dense_gather_kernel(KernelArgs da, KernelArgs ga, int n_dense,
                                                                          int dense_splits, int gather_splits,
                                                                          int gather_first, const char *k_new,
                                                                          const char *v_new)
{
    using DS = DenseSplit<D, G, kBlock, HGCA_DG_UNROLL, LD>;   // LDS sized for window splits of up to LD tokens
    using GS = SplitValu<bf16_t, D, 1, GMODE, HGCA_DG_GATHER_UNROLL>;
    constexpr int kLds = DS::kLdsBytes > GS::kLdsBytes ? DS::kLdsBytes : GS::kLdsBytes;
    __shared__ __attribute__((aligned(16))) char s_lds[kLds];
    // the part with more bytes to move takes the lower block numbers and starts first (the other fills in behind it)
    const int n_gather = (int)gridDim.x - n_dense;
    const bool dense_role = gather_first ? (int)blockIdx.x >= n_gather : (int)blockIdx.x < n_dense;
    const int u = (int)blockIdx.x - (dense_role ? (gather_first ? n_gather : 0) : (gather_first ? 0 : n_dense));
    if (dense_role) {                            // uniform over the workgroup
        const int split = u % dense_splits, kvh = (u / dense_splits) % da.sh.n_kv_heads,
                  b = u / (dense_splits * da.sh.n_kv_heads);
        int n = tier_len(da.kv, b);
        const int t0 = split * da.chunk;
        if (k_new) {                             // uniform over the launch: the window takes one more token first
            const int len = da.kv.seq_lens[b], first = da.kv.first_block[b];
            const int grown = pending_window_len(len, first, 1, da.kv.cap, da.kv.block_size, da.kv.max_blocks, nullptr);
            n = min(max(grown, 0), da.kv.cap);
            if (grown > len && len >= t0 && len < t0 + da.chunk) {
                // this split owns the token's position: its K and V rows go into the window's block, then the split
                // reads them back like any other row (no other workgroup of the launch touches that position)
                constexpr int kPieces = D * 2 / 16, kRow = D * 2;
                if (threadIdx.x < 2 * kPieces) {
                    const bool is_v = threadIdx.x >= kPieces;
                    const int piece = threadIdx.x % kPieces;
                    const int64_t blk = da.kv.block_table[(int64_t)b * da.kv.max_blocks + first + len / da.kv.block_size];
                    const int64_t dst = ((blk * da.sh.n_kv_heads + kvh) * da.kv.block_size + len % da.kv.block_size) * kRow;
                    const int64_t src = ((int64_t)b * da.sh.n_kv_heads + kvh) * kRow;
                    *reinterpret_cast<uint4 *>(const_cast<char *>(is_v ? da.kv.v : da.kv.k) + dst + 16 * piece) =
                        *reinterpret_cast<const uint4 *>((is_v ? v_new : k_new) + src + 16 * piece);
                }
                __syncthreads();
            }
        }
        if (t0 >= n) {
            write_empty_partial<D, G>(da.part, (int64_t)b * da.sh.n_q_heads + (int64_t)kvh * G, split);
            return;
        }
        DS::run(da, s_lds, split, kvh, b, t0, min(da.chunk, n - t0));
        return;
    }
    GS::run(ga, s_lds, u % gather_splits, (u / gather_splits) % ga.sh.n_q_heads, u / (gather_splits * ga.sh.n_q_heads));
}

}  // namespace

bool dense_gather_fusable(int dtype, int head_dim, int group)
{
    return dtype == 1 && (head_dim == 64 || head_dim == 128) && (group == 1 || group == 2 || group == 4);
}

hipError_t launch_dense_gather(int dtype, int head_dim, const AttnArgs &dense, const AttnArgs &gather, hipStream_t s,
                               const void *k_new, const void *v_new)
{
    if (!dense_gather_fusable(dtype, head_dim, dense.sh.group) || gather.grouped) return hipErrorInvalidValue;
    if ((k_new != nullptr) != (v_new != nullptr)) return hipErrorInvalidValue;
    if (k_new && (!dense.kv.block_table || !dense.kv.first_block || !dense.kv.seq_lens)) return hipErrorInvalidValue;
    const int64_t n_dense = (int64_t)dense.sh.batch * dense.sh.n_kv_heads * dense.part.n_splits;
    const int64_t n_gather = (int64_t)gather.sh.batch * gather.sh.n_q_heads * gather.part.n_splits;
    if (n_dense + n_gather == 0) return hipSuccess;
    if (n_dense + n_gather > 0x7fffffff) return hipErrorInvalidValue;
    auto to_ka = [](const AttnArgs &a) {
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
    };
    const KernelArgs da = to_ka(dense), ga = to_ka(gather);
    const dim3 grid((unsigned)(n_dense + n_gather)), block(kBlock);
    const int g = dense.sh.group;
    // the window's splits size the launch's LDS: the common 256-token splits leave room for seven workgroups per unit
#define HGCA_DG_LAUNCH(D, G, GMODE, LD, FIRST)                                                                      \
    hipLaunchKernelGGL((dense_gather_kernel<D, G, GMODE, LD>), grid, block, 0, s, da, ga, (int)n_dense,             \
                       dense.part.n_splits, gather.part.n_splits, FIRST, static_cast<const char *>(k_new),        \
                       static_cast<const char *>(v_new))
#define HGCA_DG_CASE(D, G)                                                                                          \
    if (head_dim == D && g == G) {                                                                                  \
        if (gather.sel_scores) {                                                                                    \
            if (dense.chunk <= 256) HGCA_DG_LAUNCH(D, G, kGatherScored, 256, 0);                                    \
            else HGCA_DG_LAUNCH(D, G, kGatherScored, kMaxChunk, 0);                                                 \
        } else {                                                                                                    \
            if (dense.chunk <= 256) HGCA_DG_LAUNCH(D, G, kGather, 256, 1);                                          \
            else HGCA_DG_LAUNCH(D, G, kGather, kMaxChunk, 1);                                                       \
        }                                                                                                           \
        return hipGetLastError();                                                                                   \
    }
    HGCA_DG_CASE(64, 1) HGCA_DG_CASE(64, 2) HGCA_DG_CASE(64, 4)
    HGCA_DG_CASE(128, 1) HGCA_DG_CASE(128, 2) HGCA_DG_CASE(128, 4)
#undef HGCA_DG_CASE
#undef HGCA_DG_LAUNCH
    return hipErrorInvalidValue;
}

}  // namespace hgca
