/*
 * CPU oracle, compiled form: the token-by-token recurrence of causal linear
 * attention with decay, in fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  Shares no code with the GPU library and is never
 * linked into it.  Used by the tests, the smoke check and the benchmark's CPU
 * baseline leg.
 *
 * What it computes, for each independent scan s = 0..S-1 (one (batch, head)
 * pair) over x[s] of shape [n, d] with decay lam[s]:
 *
 *   forward (Alg. 2; with decay, App. A second equation block; App. C
 *   "Forward Pass"):
 *       kv_0 = 0 ; kv_t = lam * kv_{t-1} + k_t v_t^T ; o_t^T = q_t^T kv_t
 *
 *   backward (Sec. 3.2 last display; with decay, App. C "Backward Pass"):
 *       dq_t^T = do_t^T kv_t^T
 *       dkv_{n+1} = 0 ; dkv_t = lam * dkv_{t+1} + q_t do_t^T
 *       dk_t^T = v_t^T dkv_t^T ; dv_t^T = k_t^T dkv_t
 *
 * kv and dkv are d x d, rows = key feature i, cols = value feature j.
 * No blocking, no reordering: one token at a time, in the order written.
 * OpenMP runs different scans on different threads; a scan is sequential.
 */
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int la_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Q,K,V,O: [S, n, d] fp64 contiguous; lam: [S]. Returns 0, or -1 on OOM. */
int la_oracle_recurrence_fwd(const double *Q, const double *K, const double *V,
                             const double *lam, double *O,
                             long S, long n, long d)
{
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long s = 0; s < S; ++s) {
        double *kv = (double *)calloc((size_t)(d * d), sizeof(double));
        if (!kv) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        const double l = lam[s];
        for (long t = 0; t < n; ++t) {
            const double *q = Q + (s * n + t) * d;
            const double *k = K + (s * n + t) * d;
            const double *v = V + (s * n + t) * d;
            double *o = O + (s * n + t) * d;
            for (long i = 0; i < d; ++i)
                for (long j = 0; j < d; ++j)
                    kv[i * d + j] = l * kv[i * d + j] + k[i] * v[j];
            for (long j = 0; j < d; ++j) o[j] = 0.0;
            for (long i = 0; i < d; ++i)
                for (long j = 0; j < d; ++j)
                    o[j] += q[i] * kv[i * d + j];
        }
        free(kv);
    }
    return fail ? -1 : 0;
}

/* Q,K,V,dO,dQ,dK,dV: [S, n, d] fp64 contiguous; lam: [S]. */
int la_oracle_recurrence_bwd(const double *Q, const double *K, const double *V,
                             const double *lam, const double *dO,
                             double *dQ, double *dK, double *dV,
                             long S, long n, long d)
{
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long s = 0; s < S; ++s) {
        double *kv = (double *)calloc((size_t)(d * d), sizeof(double));
        if (!kv) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        const double l = lam[s];
        /* forward scan: dq_t = kv_t do_t */
        for (long t = 0; t < n; ++t) {
            const double *k = K + (s * n + t) * d;
            const double *v = V + (s * n + t) * d;
            const double *g = dO + (s * n + t) * d;
            double *dq = dQ + (s * n + t) * d;
            for (long i = 0; i < d; ++i)
                for (long j = 0; j < d; ++j)
                    kv[i * d + j] = l * kv[i * d + j] + k[i] * v[j];
            for (long i = 0; i < d; ++i) {
                double acc = 0.0;
                for (long j = 0; j < d; ++j) acc += kv[i * d + j] * g[j];
                dq[i] = acc;
            }
        }
        /* reverse scan: dkv_t, dk_t = dkv_t v_t, dv_t = dkv_t^T k_t */
        memset(kv, 0, (size_t)(d * d) * sizeof(double));
        double *dkv = kv;
        for (long t = n - 1; t >= 0; --t) {
            const double *q = Q + (s * n + t) * d;
            const double *k = K + (s * n + t) * d;
            const double *v = V + (s * n + t) * d;
            const double *g = dO + (s * n + t) * d;
            double *dk = dK + (s * n + t) * d;
            double *dv = dV + (s * n + t) * d;
            for (long i = 0; i < d; ++i)
                for (long j = 0; j < d; ++j)
                    dkv[i * d + j] = l * dkv[i * d + j] + q[i] * g[j];
            for (long i = 0; i < d; ++i) {
                double acc = 0.0;
                for (long j = 0; j < d; ++j) acc += dkv[i * d + j] * v[j];
                dk[i] = acc;
            }
            for (long j = 0; j < d; ++j) dv[j] = 0.0;
            for (long i = 0; i < d; ++i)
                for (long j = 0; j < d; ++j)
                    dv[j] += k[i] * dkv[i * d + j];
        }
        free(kv);
    }
    return fail ? -1 : 0;
}
