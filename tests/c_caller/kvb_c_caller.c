/*
 * A caller of the kvb C ABI written in plain C99: device memory from hipMalloc, no Python, no
 * PyTorch, no C++.  It decodes a few chunks of a small batch with kvb_decode_flush, verifies
 * three drafts with kvb_verify, commits two of them with kvb_flush, and compares outputs and the
 * final state with the fp64 recurrence of oracle/gdn_oracle.c (test infrastructure, linked here
 * as a test may) on the same inputs.  Exit status 0 = everything within the bound.
 *
 * Inputs are bf16-exact by construction (small integers over a power of two), so the fp32
 * host arrays, their bf16 device copies and the oracle's fp64 copies hold the same values.
 *
 * Built by tests/c_caller/build.py (gcc; links libkvb.so, libgdn_oracle.so and the HIP runtime).
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kvb.h"

int gdn_oracle_sequence(int B, int T, int Hk, int Hv, int dk, int dv, const int *len, double scale, double *S,
                        const double *q, const double *k, const double *v, const double *g, const double *beta,
                        double *o, double *u, int nthreads);

enum { B = 3, HK = 2, HV = 4, D = 128, C = 4, NDEC = 10, NDRAFT = 3, NACC = 2, CAP = C - 1 + NDRAFT, T = NDEC + NDRAFT };

#define CHECK_HIP(x)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                      \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define CHECK_KVB(x)                                                                     \
    do {                                                                                 \
        int r_ = (x);                                                                    \
        if (r_ != KVB_OK) {                                                              \
            fprintf(stderr, "%s: %s\n", #x, kvb_strerror(r_));                           \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

static uint32_t lcg_state = 12345u;
static int lcg(int lo, int hi) /* uniform integer in lo..hi */
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return lo + (int)((lcg_state >> 8) % (uint32_t)(hi - lo + 1));
}

static uint16_t to_bf16(float x) /* exact for the values used here */
{
    uint32_t w;
    memcpy(&w, &x, 4);
    return (uint16_t)(w >> 16);
}

/* [B, n, H, D] fp32 host rows t0 .. t0+n-1 of a [B, T, H, D] array, as bf16 on the device */
static int upload_bf16(void *dst, const float *src, int H, int t0, int n)
{
    const size_t row = (size_t)H * D;
    uint16_t *tmp = (uint16_t *)malloc((size_t)B * n * row * 2);
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < n; ++t)
            for (size_t e = 0; e < row; ++e)
                tmp[((size_t)b * n + t) * row + e] = to_bf16(src[((size_t)b * T + t0 + t) * row + e]);
    hipError_t e = hipMemcpy(dst, tmp, (size_t)B * n * row * 2, hipMemcpyHostToDevice);
    free(tmp);
    return e == hipSuccess ? 0 : 1;
}
static int upload_f32(void *dst, const float *src, int t0, int n) /* [B, n, HV] rows of a [B, T, HV] array */
{
    float *tmp = (float *)malloc((size_t)B * n * HV * 4);
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < n; ++t)
            for (int h = 0; h < HV; ++h)
                tmp[((size_t)b * n + t) * HV + h] = src[((size_t)b * T + t0 + t) * HV + h];
    hipError_t e = hipMemcpy(dst, tmp, (size_t)B * n * HV * 4, hipMemcpyHostToDevice);
    free(tmp);
    return e == hipSuccess ? 0 : 1;
}

static double rel_err(const float *got, const double *want, size_t n)
{
    double ss = 0.0, worst = 0.0;
    for (size_t i = 0; i < n; ++i) {
        ss += want[i] * want[i];
        const double e = fabs((double)got[i] - want[i]);
        if (e > worst)
            worst = e;
    }
    return worst / sqrt(ss / (double)n + 1e-300);
}

int main(void)
{
    const size_t nqk = (size_t)B * T * HK * D, nv = (size_t)B * T * HV * D, ng = (size_t)B * T * HV;
    float *q = (float *)malloc(nqk * 4), *k = (float *)malloc(nqk * 4), *v = (float *)malloc(nv * 4);
    float *g = (float *)malloc(ng * 4), *beta = (float *)malloc(ng * 4);
    for (size_t i = 0; i < nqk; ++i) {
        q[i] = (float)lcg(-8, 8) / 64.0f;
        k[i] = (float)lcg(-8, 8) / 64.0f; /* |k|^2 about 0.75: a contraction for every beta <= 1 */
    }
    for (size_t i = 0; i < nv; ++i)
        v[i] = (float)lcg(-96, 96) / 32.0f;
    for (size_t i = 0; i < ng; ++i) {
        g[i] = -(float)lcg(0, 32) / 64.0f;
        beta[i] = (float)lcg(8, 60) / 64.0f;
    }

    if (kvb_version() != KVB_VERSION) {
        fprintf(stderr, "library version %d, header %d\n", kvb_version(), KVB_VERSION);
        return 1;
    }

    /* the store: state, record buffers, fill and status words, all owned by this caller */
    kvb_store st;
    memset(&st, 0, sizeof st);
    const size_t state_bytes = (size_t)B * HV * D * D * 4;
    void *d_slot, *d_q, *d_k, *d_v, *d_g, *d_beta, *d_out, *d_acc;
    CHECK_HIP(hipMalloc((void **)&st.state, state_bytes));
    CHECK_HIP(hipMalloc(&st.buf_k, (size_t)B * HK * CAP * D * 2));
    CHECK_HIP(hipMalloc(&st.buf_u, (size_t)B * HV * CAP * D * 4));
    CHECK_HIP(hipMalloc((void **)&st.buf_G, (size_t)B * HV * CAP * 4));
    CHECK_HIP(hipMalloc((void **)&st.fill, B * 4));
    CHECK_HIP(hipMalloc((void **)&st.status, B * 4));
    CHECK_HIP(hipMemset(st.state, 0, state_bytes));
    CHECK_HIP(hipMemset(st.fill, 0, B * 4));
    CHECK_HIP(hipMemset(st.status, 0, B * 4));
    st.n_slots = B;
    CHECK_HIP(hipMalloc(&d_slot, B * 4));
    CHECK_HIP(hipMalloc(&d_acc, B * 4));
    CHECK_HIP(hipMalloc(&d_q, (size_t)B * NDRAFT * HK * D * 2));
    CHECK_HIP(hipMalloc(&d_k, (size_t)B * NDRAFT * HK * D * 2));
    CHECK_HIP(hipMalloc(&d_v, (size_t)B * NDRAFT * HV * D * 2));
    CHECK_HIP(hipMalloc(&d_g, (size_t)B * NDRAFT * HV * 4));
    CHECK_HIP(hipMalloc(&d_beta, (size_t)B * NDRAFT * HV * 4));
    CHECK_HIP(hipMalloc(&d_out, (size_t)B * NDRAFT * HV * D * 4));
    int32_t slot[B], acc[B];
    for (int b = 0; b < B; ++b) {
        slot[b] = B - 1 - b; /* any permutation */
        acc[b] = NACC;
    }
    CHECK_HIP(hipMemcpy(d_slot, slot, sizeof slot, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_acc, acc, sizeof acc, hipMemcpyHostToDevice));

    kvb_shape sh;
    memset(&sh, 0, sizeof sh);
    sh.B = B; sh.Hk = HK; sh.Hv = HV; sh.dk = D; sh.dv = D; sh.cap = CAP;
    sh.in_dtype = KVB_BF16; sh.out_dtype = KVB_F32; sh.rec_dtype = KVB_F32; sh.scale = 1.0f;

    float *out = (float *)malloc(nv * 4); /* [B, T, HV, D] as the oracle lays it out */
    float *step = (float *)malloc((size_t)B * NDRAFT * HV * D * 4);
    /* chunkwise decoding, one token per call, the state folded every C tokens in the same kernel */
    for (int t = 0; t < NDEC; ++t) {
        if (upload_bf16(d_q, q, HK, t, 1) || upload_bf16(d_k, k, HK, t, 1) || upload_bf16(d_v, v, HV, t, 1) ||
            upload_f32(d_g, g, t, 1) || upload_f32(d_beta, beta, t, 1))
            return 2;
        CHECK_KVB(kvb_decode_flush(&sh, &st, (const int32_t *)d_slot, d_q, d_k, d_v, (const float *)d_g,
                                   (const float *)d_beta, d_out, C, NULL));
        CHECK_HIP(hipMemcpy(step, d_out, (size_t)B * HV * D * 4, hipMemcpyDeviceToHost));
        for (int b = 0; b < B; ++b)
            memcpy(out + ((size_t)b * T + t) * HV * D, step + (size_t)b * HV * D, (size_t)HV * D * 4);
    }
    /* three drafts in one call; two are accepted and folded into the state */
    if (upload_bf16(d_q, q, HK, NDEC, NDRAFT) || upload_bf16(d_k, k, HK, NDEC, NDRAFT) ||
        upload_bf16(d_v, v, HV, NDEC, NDRAFT) || upload_f32(d_g, g, NDEC, NDRAFT) || upload_f32(d_beta, beta, NDEC, NDRAFT))
        return 2;
    CHECK_KVB(kvb_verify(&sh, &st, (const int32_t *)d_slot, NDRAFT, d_q, d_k, d_v, (const float *)d_g,
                         (const float *)d_beta, d_out, NULL));
    CHECK_KVB(kvb_flush(&sh, &st, (const int32_t *)d_slot, (const int32_t *)d_acc, 1, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(step, d_out, (size_t)B * NDRAFT * HV * D * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b)
        memcpy(out + ((size_t)b * T + NDEC) * HV * D, step + (size_t)b * NDRAFT * HV * D, (size_t)NDRAFT * HV * D * 4);
    float *state = (float *)malloc(state_bytes);
    int32_t fill[B], status[B];
    CHECK_HIP(hipMemcpy(state, st.state, state_bytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(fill, st.fill, sizeof fill, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(status, st.status, sizeof status, hipMemcpyDeviceToHost));

    /* the oracle: all T tokens for the outputs, the first NDEC + NACC for the committed state */
    double *qd = (double *)malloc(nqk * 8), *kd = (double *)malloc(nqk * 8), *vd = (double *)malloc(nv * 8);
    double *gd = (double *)malloc(ng * 8), *bd = (double *)malloc(ng * 8), *od = (double *)malloc(nv * 8);
    double *S = (double *)calloc((size_t)B * HV * D * D, 8);
    for (size_t i = 0; i < nqk; ++i) { qd[i] = q[i]; kd[i] = k[i]; }
    for (size_t i = 0; i < nv; ++i) vd[i] = v[i];
    for (size_t i = 0; i < ng; ++i) { gd[i] = g[i]; bd[i] = beta[i]; }
    if (gdn_oracle_sequence(B, T, HK, HV, D, D, NULL, 1.0, S, qd, kd, vd, gd, bd, od, NULL, 0) < 0)
        return 4;
    const double e_out = rel_err(out, od, nv);
    int len[B];
    for (int b = 0; b < B; ++b)
        len[b] = NDEC + NACC;
    memset(S, 0, (size_t)B * HV * D * D * 8);
    if (gdn_oracle_sequence(B, T, HK, HV, D, D, len, 1.0, S, qd, kd, vd, gd, bd, od, NULL, 0) < 0)
        return 4;
    /* request b lives in slot[b] */
    double worst_state = 0.0;
    for (int b = 0; b < B; ++b) {
        const double e = rel_err(state + (size_t)slot[b] * HV * D * D, S + (size_t)b * HV * D * D, (size_t)HV * D * D);
        if (e > worst_state)
            worst_state = e;
    }
    int bad = 0;
    for (int b = 0; b < B; ++b)
        bad |= fill[b] != 0 || status[b] != 0;
    printf("kvb_c_caller: rel err outputs %.2e, committed state %.2e, fill/status clean: %s\n", e_out, worst_state,
           bad ? "no" : "yes");
    const double bound = 2e-4; /* fp32 arithmetic on exact inputs: observed about 1e-6 */
    return (e_out < bound && worst_state < bound && !bad) ? 0 : 1;
}
