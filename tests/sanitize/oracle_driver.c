/*
 * Host-side sanitizer driver for the compiled oracle (tests/test_sanitizers_cpu.py builds this
 * file together with oracle/la_oracle.c under -fsanitize=address,undefined and runs it).
 * It calls both entry points on exactly-sized heap buffers, for several shapes including
 * d = 1, n = 1 and more scans than threads, and checks worked example A of the test-suite
 * (d = 1, n = 3, lambda = 0.5): any out-of-bounds access, use of uninitialised heap memory
 * that ASan can see, signed overflow or misaligned access aborts the run.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int la_oracle_recurrence_fwd(const double *Q, const double *K, const double *V, const double *lam, double *O,
                             long S, long n, long d);
int la_oracle_recurrence_bwd(const double *Q, const double *K, const double *V, const double *lam,
                             const double *dO, double *dQ, double *dK, double *dV, long S, long n, long d);

static double *filled(size_t count, unsigned seed)
{
    double *p = (double *)malloc(count * sizeof(double));
    if (!p) exit(2);
    for (size_t i = 0; i < count; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = ((double)(seed >> 8) / 16777216.0) - 0.5;
    }
    return p;
}

static int run_shape(long S, long n, long d)
{
    const size_t el = (size_t)(S * n * d);
    double *q = filled(el, 1), *k = filled(el, 2), *v = filled(el, 3), *g = filled(el, 4);
    double *lam = (double *)malloc((size_t)S * sizeof(double));
    double *o = (double *)malloc(el * sizeof(double)), *dq = (double *)malloc(el * sizeof(double));
    double *dk = (double *)malloc(el * sizeof(double)), *dv = (double *)malloc(el * sizeof(double));
    if (!lam || !o || !dq || !dk || !dv) exit(2);
    for (long s = 0; s < S; ++s) lam[s] = 1.0 - 0.1 * (double)(s % 7);
    int rc = la_oracle_recurrence_fwd(q, k, v, lam, o, S, n, d);
    rc |= la_oracle_recurrence_bwd(q, k, v, lam, g, dq, dk, dv, S, n, d);
    double sum = 0.0;
    for (size_t i = 0; i < el; ++i) sum += o[i] + dq[i] + dk[i] + dv[i];
    free(q); free(k); free(v); free(g); free(lam); free(o); free(dq); free(dk); free(dv);
    if (rc != 0 || !isfinite(sum)) {
        fprintf(stderr, "shape S=%ld n=%ld d=%ld failed (rc=%d)\n", S, n, d, rc);
        return 1;
    }
    return 0;
}

int main(void)
{
    int bad = 0;
    const long shapes[][3] = {{1, 1, 1}, {1, 3, 1}, {3, 17, 5}, {40, 9, 8}, {2, 130, 64}, {1, 33, 128}};
    for (size_t i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i)
        bad |= run_shape(shapes[i][0], shapes[i][1], shapes[i][2]);
    /* worked example A: q = (1,2,3), k = (1,1,2), v = (1,2,3), dO = (1,1,1), lambda = 0.5 */
    const double q[3] = {1, 2, 3}, k[3] = {1, 1, 2}, v[3] = {1, 2, 3}, g[3] = {1, 1, 1}, lam[1] = {0.5};
    double o[3], dq[3], dk[3], dv[3];
    bad |= la_oracle_recurrence_fwd(q, k, v, lam, o, 1, 3, 1);
    bad |= la_oracle_recurrence_bwd(q, k, v, lam, g, dq, dk, dv, 1, 3, 1);
    const double want_o[3] = {1, 5, 21.75}, want_dk[3] = {2.75, 7, 9};
    for (int t = 0; t < 3; ++t)
        if (fabs(o[t] - want_o[t]) > 1e-12 || fabs(dk[t] - want_dk[t]) > 1e-12) bad = 1;
    if (bad) {
        fprintf(stderr, "oracle sanitizer driver: FAILED\n");
        return 1;
    }
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
