// Device-side helpers shared by the HGCA kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hgca {

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage tag: upper half of an IEEE fp32

// One KV tier as the kernels see it (mirrors hgca_kv_view, pointers are device memory).
struct KvDev {
    const char *k, *v;
    const int32_t *seq_lens;
    const int32_t *block_table;
    const int32_t *first_block;     // paged only: per-sequence offset into the table row, or null
    int32_t cap, block_size, max_blocks;
    // N queries per sequence on a path written for one: batch index bv of the launch stands for query bv % n_q of
    // sequence bv / n_q (n_q <= 1: off).  With causal_tail the tier's last n_q valid tokens are the queries' own and
    // query i sees the tokens before position len - n_q + i + 1.
    int32_t n_q, causal_tail;
};

// Shape scalars passed by value to kernels.
struct ShapeDev {
    int32_t batch, n_q_heads, n_kv_heads, group;
    float sm_scale;
};

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int kPerLoad = 4;            // elements in one 16-byte load
    static __device__ __forceinline__ void expand(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};

template <> struct Elem<bf16_t> {
    static constexpr int kPerLoad = 8;
    static __device__ __forceinline__ void expand(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
};

// The sequence whose K/V rows batch index b of a launch reads.
__device__ __forceinline__ int kv_seq(const KvDev &kv, int b) { return kv.n_q > 1 ? b / kv.n_q : b; }

__device__ __forceinline__ int32_t tier_len(const KvDev &kv, int b) {
    const int seq = kv_seq(kv, b);
    const int32_t len = kv.seq_lens ? min(max(kv.seq_lens[seq], 0), kv.cap) : kv.cap;   // never beyond the buffer
    if (kv.n_q > 1 && kv.causal_tail) return min(max(len - kv.n_q + (b - seq * kv.n_q) + 1, 0), len);
    return len;
}

__device__ __forceinline__ uint4 load16(const char *p) {
    return *reinterpret_cast<const uint4 *>(p);
}

// 16-byte load marked non-temporal: K/V rows are streamed once and should not displace
// reusable lines in the caches.
__device__ __forceinline__ uint4 load16_stream(const char *p) {
    const uint32_t *w = reinterpret_cast<const uint32_t *>(p);
    uint4 r;
    r.x = __builtin_nontemporal_load(w + 0);
    r.y = __builtin_nontemporal_load(w + 1);
    r.z = __builtin_nontemporal_load(w + 2);
    r.w = __builtin_nontemporal_load(w + 3);
    return r;
}

template <int kWidth>
__device__ __forceinline__ float group_sum(float v) {      // sum over kWidth adjacent lanes
#pragma unroll
    for (int off = kWidth / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

}  // namespace hgca
