/*
 * TEST INFRASTRUCTURE -- the parity oracle.  Not part of the product path.
 *
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg may
 * build, load or call this file.  It shares nothing with the HIP library.
 *
 * What it computes: the token-by-token recurrent form of Gated DeltaNet
 * (paper App. A.1, Eq. 11-12), with the output rule o_t = q_t S_t of the
 * recurrent form (Sec. 2.1, Eq. 3), in fp64, for every (request, v-head)
 * unit independently:
 *
 *     S~  = alpha_t * S_{t-1}                     alpha_t = exp(g_t)     (Eq. 11)
 *     S_t = S~ - beta_t k_t^T (k_t S~) + beta_t k_t^T v_t                (Eq. 12)
 *     o_t = scale * q_t S_t                                              (Eq. 3)
 *
 * Eq. 12 is evaluated through the delta value u_t = beta_t (v_t - k_t S~),
 * S_t = S~ + k_t^T u_t, which is the same expression with the two rank-one
 * terms collected; u_t is returned because the chunkwise form buffers it
 * (App. A.1, the paragraph after Eq. 16).
 *
 * Every KVBuffer call (decode, flush, verify, direct) is, by Sec. 2.1 and
 * App. A.1, an exact regrouping of this recurrence, so this is the definition
 * all four are compared against.  There is no blocking or reordering here.
 *
 * Grouped heads: v-head h reads the q and k of qk-head h / (Hv / Hk).
 *
 * Parity pins: tests/test_oracle_pins.py (closed forms, dense-inverse
 * chunkwise form, linear-attention reduction, hand-worked example).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One (request, v-head) unit, n tokens.  Row strides are in elements. */
static void gdn_unit(int n, int dk, int dv, double scale, double *S,
                     const double *q, size_t sq, const double *k, size_t sk,
                     const double *v, size_t sv, const double *g, size_t sg,
                     const double *beta, size_t sb, double *o, size_t so,
                     double *u_out, size_t su, double *u)
{
    for (int t = 0; t < n; ++t) {
        const double *qt = q + (size_t)t * sq;
        const double *kt = k + (size_t)t * sk;
        const double *vt = v + (size_t)t * sv;
        const double alpha = exp(g[(size_t)t * sg]);
        const double bt = beta[(size_t)t * sb];

        /* Eq. 11: gate the whole state. */
        for (int i = 0; i < dk * dv; ++i)
            S[i] *= alpha;

        /* old value stored under this key, then the delta value */
        for (int j = 0; j < dv; ++j) {
            double r = 0.0;
            for (int i = 0; i < dk; ++i)
                r += kt[i] * S[(size_t)i * dv + j];
            u[j] = bt * (vt[j] - r);
        }

        /* Eq. 12: rank-one write */
        for (int i = 0; i < dk; ++i)
            for (int j = 0; j < dv; ++j)
                S[(size_t)i * dv + j] += kt[i] * u[j];

        /* Eq. 3: read with the query from the updated state */
        for (int j = 0; j < dv; ++j) {
            double acc = 0.0;
            for (int i = 0; i < dk; ++i)
                acc += qt[i] * S[(size_t)i * dv + j];
            o[(size_t)t * so + j] = scale * acc;
        }
        if (u_out)
            for (int j = 0; j < dv; ++j)
                u_out[(size_t)t * su + j] = u[j];
    }
}

/*
 * Batched driver.  All arrays are fp64, C-contiguous:
 *   S    [B, Hv, dk, dv]   in: state before the first token; out: after token len[b]-1
 *   q,k  [B, T, Hk, dk]    v, o, u [B, T, Hv, dv]    g, beta [B, T, Hv]
 *   len  [B] or NULL       tokens processed for request b (0..T); NULL = T for all
 *   u    may be NULL
 * Rows t >= len[b] of o and u are left untouched.
 * Returns the number of threads used, or -1 on a bad argument.
 */
int gdn_oracle_sequence(int B, int T, int Hk, int Hv, int dk, int dv,
                        const int *len, double scale, double *S,
                        const double *q, const double *k, const double *v,
                        const double *g, const double *beta, double *o,
                        double *u, int nthreads)
{
    if (B < 0 || T < 0 || Hk <= 0 || Hv <= 0 || dk <= 0 || dv <= 0 ||
        Hv % Hk != 0)
        return -1;
    const int r = Hv / Hk;
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
    used = omp_get_max_threads();
#else
    (void)nthreads;
#endif
    const long units = (long)B * Hv;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)dv);
#pragma omp for schedule(dynamic, 1)
        for (long w = 0; w < units; ++w) {
            const int b = (int)(w / Hv), h = (int)(w % Hv), hk = h / r;
            int n = len ? len[b] : T;
            if (n > T) n = T;
            if (n < 0) n = 0;
            const size_t tok_qk = (size_t)Hk * dk, tok_v = (size_t)Hv * dv;
            gdn_unit(n, dk, dv, scale,
                     S + ((size_t)b * Hv + h) * dk * dv,
                     q + (size_t)b * T * tok_qk + (size_t)hk * dk, tok_qk,
                     k + (size_t)b * T * tok_qk + (size_t)hk * dk, tok_qk,
                     v + (size_t)b * T * tok_v + (size_t)h * dv, tok_v,
                     g + (size_t)b * T * Hv + h, (size_t)Hv,
                     beta + (size_t)b * T * Hv + h, (size_t)Hv,
                     o + (size_t)b * T * tok_v + (size_t)h * dv, tok_v,
                     u ? u + (size_t)b * T * tok_v + (size_t)h * dv : NULL,
                     tok_v, tmp);
        }
        free(tmp);
    }
    return used;
}
