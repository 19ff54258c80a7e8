// Fold of split partials into one attention result (merge_state over any number of splits), as device code shared
// by the fold kernel and by kernels that go on with the row after folding it.
#pragma once

#include "hgca_launch.hpp"

namespace hgca {

constexpr int kFoldBlock = 256;                  // threads of the workgroup that folds one (b, h) row
constexpr int kFoldWaves = kFoldBlock / kWave;

template <int D> struct FoldShared {
    float4 acc[kFoldBlock / (D / 4)][D / 4];
    float L[kFoldBlock / (D / 4)];
    float M[kFoldWaves];
    float lse_p;
};

// Folds split partials of one (b, h) row: M = max m_s, L = sum l_s e^{m_s-M}, O = sum o_s e^{m_s-M} / L,
// lse = M + ln L.  The splits may come from two partial sets (p and q): folding the splits of the dense
// window part and of the sparse part in one go is merge_state applied to all of them at once
// (the fusion is associative).  Thread (sg, c4) sums the splits sg, sg+SG, ... of four adjacent columns;
// the SG groups are then added through LDS.  Called by all kFoldBlock threads of a workgroup.  With WANT_P the
// log-sum-exp of set p alone (the window part of a step: its attention weights are normalised by it) is formed by
// the last wave, stored to lse_p[row] if lse_p is given, and returned to every thread; otherwise 0 is returned.
// lse_q (with WANT_P only) receives the same for set q.
template <int D, bool OUT_BF16, bool WANT_P>
__device__ __forceinline__ float fold_row(FoldShared<D> &sh, const Partials &p, const Partials &q, void *o, float *lse,
                                          float *lse_p, int64_t row, float *lse_q = nullptr)
{
    constexpr int C4 = D / 4;                    // threads across the columns (one float4 each)
    constexpr int SG = kFoldBlock / C4;          // split groups
    constexpr int PRE = 4;                       // splits per thread whose loads are issued before anything is used

    const int tid = threadIdx.x, sg = tid / C4, c4 = tid % C4;
    const int np = p.n_splits, n = np + q.n_splits;
    auto m_of = [&](int s) { return s < np ? p.m[row * np + s] : q.m[row * q.n_splits + (s - np)]; };
    auto l_of = [&](int s) { return s < np ? p.l[row * np + s] : q.l[row * q.n_splits + (s - np)]; };
    auto o_of = [&](int s) {
        const float *base = s < np ? p.o + (row * np + s) * D : q.o + (row * q.n_splits + (s - np)) * D;
        return *reinterpret_cast<const float4 *>(base + 4 * c4);
    };
    // One round trip to memory for the usual split counts: a thread's first PRE splits (m, l and its four columns
    // of o) are requested together with the maxima it contributes to the row's maximum; the weights e^{m-M} need
    // M, but the loads do not.
    float pm[PRE], pl[PRE];
    float4 po[PRE];
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const int s = sg + i * SG;
        pm[i] = -INFINITY;
        pl[i] = 0.f;
        po[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s < n) { pm[i] = m_of(s); pl[i] = l_of(s); po[i] = o_of(s); }
    }
    // the maximum over all splits: one split per thread, then over the workgroup
    float M = -INFINITY;
    for (int s = tid; s < n; s += kFoldBlock) M = fmaxf(M, m_of(s));
    M = wave_max(M);
    if (tid % kWave == 0) sh.M[tid / kWave] = M;
    // set p alone, on the last wave: a lane per split, fixed reduction order
    if (WANT_P && tid / kWave == kFoldWaves - 1) {
        const int lane = tid % kWave;
        float Mp = -INFINITY;
        for (int s = lane; s < np; s += kWave) Mp = fmaxf(Mp, p.m[row * np + s]);
        Mp = wave_max(Mp);
        float Lp = 0.f;
        if (Mp != -INFINITY)
            for (int s = lane; s < np; s += kWave) Lp = fmaf(p.l[row * np + s], expf(p.m[row * np + s] - Mp), Lp);
        Lp = wave_sum(Lp);
        if (lane == 0) {
            const float v = (Mp != -INFINITY) ? Mp + logf(Lp) : -INFINITY;
            sh.lse_p = v;
            if (lse_p) lse_p[row] = v;
        }
    }
    // set q alone, on the wave before the last, if asked for (uniform over the launch)
    if (WANT_P && lse_q && tid / kWave == kFoldWaves - 2) {
        const int lane = tid % kWave, nq = q.n_splits;
        float Mq = -INFINITY;
        for (int s = lane; s < nq; s += kWave) Mq = fmaxf(Mq, q.m[row * nq + s]);
        Mq = wave_max(Mq);
        float Lq = 0.f;
        if (Mq != -INFINITY)
            for (int s = lane; s < nq; s += kWave) Lq = fmaf(q.l[row * nq + s], expf(q.m[row * nq + s] - Mq), Lq);
        Lq = wave_sum(Lq);
        if (lane == 0) lse_q[row] = (Mq != -INFINITY) ? Mq + logf(Lq) : -INFINITY;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kFoldWaves; ++w) M = fmaxf(M, sh.M[w]);
    float L = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (M != -INFINITY) {                        // else every split is empty (uniform over the workgroup)
#pragma unroll
        for (int i = 0; i < PRE; ++i) {
            const float wgt = expf(pm[i] - M);   // 0 for empty splits and for splits beyond n (m = -inf)
            L = fmaf(pl[i], wgt, L);
            acc.x = fmaf(po[i].x, wgt, acc.x); acc.y = fmaf(po[i].y, wgt, acc.y);
            acc.z = fmaf(po[i].z, wgt, acc.z); acc.w = fmaf(po[i].w, wgt, acc.w);
        }
        for (int s = sg + PRE * SG; s < n; s += SG) {
            const float wgt = expf(m_of(s) - M);
            const float4 v = o_of(s);
            L = fmaf(l_of(s), wgt, L);
            acc.x = fmaf(v.x, wgt, acc.x); acc.y = fmaf(v.y, wgt, acc.y);
            acc.z = fmaf(v.z, wgt, acc.z); acc.w = fmaf(v.w, wgt, acc.w);
        }
    }
    sh.acc[sg][c4] = acc;
    if (c4 == 0) sh.L[sg] = L;
    __syncthreads();
    if (tid < C4) {
        float Lt = 0.f;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int g = 0; g < SG; ++g) {
            const float4 v = sh.acc[g][tid];
            t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
            Lt += sh.L[g];
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
    return WANT_P ? sh.lse_p : 0.f;
}

}  // namespace hgca
