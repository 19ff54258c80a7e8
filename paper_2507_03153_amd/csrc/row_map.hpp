// Row addressing of a split, shared by the attention kernels.
#pragma once

#include "hgca_device.hpp"

namespace hgca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

// LDS transpose read of 16-bit elements (ds_read_b64_tr_b16): inside a 16-lane group, lane i receives as its
// element e the element i % 4 of the four that lane 4e + i/4 points at.  So if lane j of a group points at
// columns 4(j%4) .. 4(j%4)+3 of row j/4 of a row-major tile, lane i ends up with column i of rows 0..3:
// the 8-tokens-of-one-column slice an MFMA operand needs, straight from the rows as they were loaded.
__device__ __forceinline__ short4v lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (short4v __attribute__((address_space(3))) *)(const_cast<char *>(p)));
}

// Token of a 32-token block that contraction index 8*g + i stands for in lane group g (g = lane / 16): tokens
// 4g..4g+3 of the block's first 16-token tile, then of its second one (the order in which a lane holds the
// results of two 16-token score tiles).
__device__ __forceinline__ int block_token(int g, int i) { return i < 4 ? 4 * g + i : 16 + 4 * g + (i - 4); }

// Where the rows of a split live: the number of the [d] row (counted over the whole K or V buffer of
// the tier) of the split's j-th token.  A dense split of a contiguous tier is plain arithmetic; paged
// tiers and index lists get a table in LDS, filled once per workgroup, so that neither the block table
// nor the index list is in the dependency chain of every row load of the K and V passes.
struct RowMap {
    const uint32_t *table;   // LDS; nullptr => row = base + j
    uint32_t base;
    __device__ __forceinline__ uint32_t operator()(int j) const { return table ? table[j] : base + (uint32_t)j; }
};

// `listed` (gather only) points at the split's first index.  Contains a barrier iff a table is filled;
// the condition is uniform over the workgroup.
template <bool GATHER, int BLOCK>
__device__ __forceinline__ RowMap make_row_map(uint32_t *s_row, const KvDev &kv, int n_kv_heads, int b, int kvh,
                                               int t0, int nt, const int32_t *listed)
{
    b = kv_seq(kv, b);                           // the sequence whose rows are read
    RowMap m;
    if (!GATHER && kv.block_table == nullptr) {
        m.table = nullptr;
        m.base = (uint32_t)(((int64_t)b * n_kv_heads + kvh) * kv.cap + t0);
        return m;
    }
    const int32_t *blocks = nullptr;             // the sequence's table row, from the tier's first block on
    if (kv.block_table) blocks = kv.block_table + (int64_t)b * kv.max_blocks + (kv.first_block ? kv.first_block[b] : 0);
    for (int j = threadIdx.x; j < nt; j += BLOCK) {
        // a listed position outside the tier is clamped into it: the result is then meaningless, but no address
        // outside the tier's buffers is formed (callers of a gather make sure that the tier is not empty)
        const int32_t tok = GATHER ? min(max(listed[j], 0), kv.cap - 1) : t0 + j;
        uint32_t row;
        if (blocks) {
            const int32_t blk = blocks[tok / kv.block_size];
            row = (uint32_t)(((int64_t)blk * n_kv_heads + kvh) * kv.block_size + tok % kv.block_size);
        } else {
            row = (uint32_t)(((int64_t)b * n_kv_heads + kvh) * kv.cap + tok);
        }
        s_row[j] = row;
    }
    __syncthreads();
    m.table = s_row;
    m.base = 0;
    return m;
}

}  // namespace hgca
