/* The library used from plain C, with nothing but the HIP runtime for device memory: one whole decode step
 * (paper Alg. 2, decode branch) through hgca_hybrid_decode_step on a small seeded case per dtype, checked
 * against the fp64 C oracle (linked into this test program only).  Exit code 0 = agreement.
 * Bars: fp32 inputs 1e-5; bf16 inputs 2e-4 (stated bar 2e-2); selections identical. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "hgca.h"
#include "hgca_oracle.h"

#define B 2
#define HQ 4
#define HKV 2
#define W 40
#define P 300
#define KSEL 17

static uint32_t lcg_state = 2507u;
static float lcg_uniform(void)            /* in [-1, 1) */
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)(lcg_state >> 8) / 8388608.0f - 1.0f;
}

static uint16_t to_bf16_bits(float x)     /* round to nearest even */
{
    uint32_t u;
    memcpy(&u, &x, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static void *dev_alloc(size_t bytes)
{
    void *dev = NULL;
    if (hipMalloc(&dev, bytes ? bytes : 16) != hipSuccess) { fprintf(stderr, "hipMalloc failed\n"); exit(2); }
    return dev;
}

static void *to_device(const void *host, size_t bytes)
{
    void *dev = dev_alloc(bytes);
    if (hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) { fprintf(stderr, "copy failed\n"); exit(2); }
    return dev;
}

static void *fill(size_t n, int bf16)      /* n seeded elements of the dtype */
{
    size_t i;
    if (bf16) {
        uint16_t *p = (uint16_t *)malloc(n * 2);
        for (i = 0; i < n; ++i) p[i] = to_bf16_bits(lcg_uniform());
        return p;
    } else {
        float *p = (float *)malloc(n * 4);
        for (i = 0; i < n; ++i) p[i] = lcg_uniform();
        return p;
    }
}

static int run_case(int bf16, int d, double tol)
{
    const size_t elem = bf16 ? 2 : 4;
    const int32_t w_lens[B] = {W, 23}, p_lens[B] = {P, 170};
    const float scale = 1.0f / sqrtf((float)d);
    void *q = fill((size_t)B * HQ * d, bf16);
    void *kw = fill((size_t)B * HKV * W * d, bf16), *vw = fill((size_t)B * HKV * W * d, bf16);
    void *kp = fill((size_t)B * HKV * P * d, bf16), *vp = fill((size_t)B * HKV * P * d, bf16);

    /* oracle */
    oracle_shape osh = {bf16 ? ORACLE_BF16 : ORACLE_F32, B, HQ, HKV, d, (double)scale};
    oracle_kv ow = {kw, vw, w_lens, NULL, W, 0, 0}, op = {kp, vp, p_lens, NULL, P, 0, 0};
    int32_t idx_ref[B * HQ * KSEL], cnt_ref[B * HQ];
    double *o_ref = (double *)malloc(sizeof(double) * B * HQ * d), lse_ref[B * HQ];
    if (oracle_hybrid_step(&osh, q, &ow, &op, NULL, KSEL, KSEL, 1, idx_ref, cnt_ref, o_ref, lse_ref) != 0) return 1;

    /* library */
    hgca_shape sh = {bf16 ? HGCA_BF16 : HGCA_F32, B, HQ, HKV, d, scale};
    void *d_q = to_device(q, (size_t)B * HQ * d * elem);
    hgca_kv_view win, pool;
    memset(&win, 0, sizeof(win));
    memset(&pool, 0, sizeof(pool));
    win.k = to_device(kw, (size_t)B * HKV * W * d * elem);
    win.v = to_device(vw, (size_t)B * HKV * W * d * elem);
    win.seq_lens = (const int32_t *)to_device(w_lens, sizeof(w_lens));
    win.cap = W;
    pool.k = to_device(kp, (size_t)B * HKV * P * d * elem);
    pool.v = to_device(vp, (size_t)B * HKV * P * d * elem);
    pool.seq_lens = (const int32_t *)to_device(p_lens, sizeof(p_lens));
    pool.cap = P;
    const size_t wsd_bytes = hgca_workspace_bytes(&sh, W, 0, 0), wss_bytes = hgca_workspace_bytes(&sh, 0, P, KSEL);
    void *wsd = dev_alloc(wsd_bytes), *wss = dev_alloc(wss_bytes);
    int32_t *d_idx = (int32_t *)dev_alloc(sizeof(idx_ref)), *d_cnt = (int32_t *)dev_alloc(sizeof(cnt_ref));
    float *d_o = (float *)dev_alloc(sizeof(float) * B * HQ * d), *d_lse = (float *)dev_alloc(sizeof(float) * B * HQ);

    const int rc = hgca_hybrid_decode_step(&sh, d_q, &win, &pool, NULL, KSEL, KSEL, d_idx, d_cnt, d_o, HGCA_F32, d_lse,
                                           wsd, wsd_bytes, wss, wss_bytes, NULL);
    if (rc != HGCA_OK) { fprintf(stderr, "hgca_hybrid_decode_step: %s\n", hgca_status_string(rc)); return 1; }
    if (hipDeviceSynchronize() != hipSuccess) { fprintf(stderr, "device error\n"); return 2; }

    int32_t idx[B * HQ * KSEL], cnt[B * HQ];
    float *o = (float *)malloc(sizeof(float) * B * HQ * d), lse[B * HQ];
    if (hipMemcpy(idx, d_idx, sizeof(idx), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(cnt, d_cnt, sizeof(cnt), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(o, d_o, sizeof(float) * B * HQ * d, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(lse, d_lse, sizeof(lse), hipMemcpyDeviceToHost) != hipSuccess)
        return 2;

    int bad = 0, i;
    double err_o = 0.0, err_l = 0.0;
    if (memcmp(cnt, cnt_ref, sizeof(cnt)) != 0 || memcmp(idx, idx_ref, sizeof(idx)) != 0) { fprintf(stderr, "selection differs\n"); bad = 1; }
    for (i = 0; i < B * HQ * d; ++i) err_o = fmax(err_o, fabs((double)o[i] - o_ref[i]));
    for (i = 0; i < B * HQ; ++i) err_l = fmax(err_l, fabs((double)lse[i] - lse_ref[i]));
    printf("abi_step %s d=%d: max|dO|=%.3e max|dlse|=%.3e (bar %.0e)%s\n", bf16 ? "bf16" : "f32", d, err_o, err_l, tol,
           bad ? " SELECTION DIFFERS" : "");
    if (!(err_o <= tol) || !(err_l <= tol)) bad = 1;
    return bad;
}

int main(void)
{
    int bad = run_case(0, 64, 1e-5);
    bad |= run_case(1, 128, 2e-4);
    if (!bad) printf("abi_step: ok\n");
    return bad;
}
