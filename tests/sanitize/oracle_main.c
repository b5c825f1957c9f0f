/* Drives the fp64 oracle on a small packed batch under AddressSanitizer and UndefinedBehaviorSanitizer
 * (built and run by tests/test_sanitizers_host.py).  Empty, one-token, ragged and multi-checkpoint sequences,
 * d_k != d_v, with and without the optional states.  Exit status 0 and no sanitizer report = pass. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int dn_oracle_fwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k, const double *v,
                  const double *beta, const double *S0, double *o, double *ST, int nthreads);
int dn_oracle_bwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k, const double *v,
                  const double *beta, const double *S0, const double *d_o, const double *dST, double *dq, double *dkk,
                  double *dvv, double *dbeta, double *dS0, int nthreads);
int dn_oracle_gated_fwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k, const double *v,
                        const double *beta, const double *g, const double *S0, double *o, double *ST, int nthreads);
int dn_oracle_gated_bwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k, const double *v,
                        const double *beta, const double *g, const double *S0, const double *d_o, const double *dST,
                        double *dq, double *dkk, double *dvv, double *dbeta, double *dg, double *dS0, int nthreads);

static uint64_t rng = 88172645463325252ull;
static double unif(void) { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (double)(rng >> 11) / 9007199254740992.0 - 0.5; }
static double *vec(size_t n, double scale) {
    double *p = (double *)malloc((n ? n : 1) * sizeof(double)); /* exact size: an overrun is a sanitizer report */
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = scale * unif();
    return p;
}

int main(void) {
    enum { N = 5, H = 2, DK = 6, DV = 5 };
    const int32_t cu[N + 1] = {0, 0, 1, 70, 133, 330}; /* the last one spans four 64-token checkpoints */
    const size_t T = 330, st = (size_t)N * H * DK * DV;
    double *q = vec(T * H * DK, 1.0), *k = vec(T * H * DK, 1.0), *v = vec(T * H * DV, 2.0), *beta = vec(T * H, 1.0);
    double *g = vec(T * H, 0.2), *d_o = vec(T * H * DV, 2.0), *S0 = vec(st, 0.1), *dST = vec(st, 1.0);
    for (size_t i = 0; i < T * H; ++i) { beta[i] += 0.5; g[i] = -fabs(g[i]); }
    double *o = vec(T * H * DV, 0), *ST = vec(st, 0), *dq = vec(T * H * DK, 0), *dk = vec(T * H * DK, 0), *dv = vec(T * H * DV, 0);
    double *db = vec(T * H, 0), *dg = vec(T * H, 0), *dS0 = vec(st, 0);
    int rc = 0;
    for (int pass = 0; pass < 2; ++pass) {
        const double *s0 = pass ? S0 : NULL, *dst = pass ? dST : NULL;
        rc |= dn_oracle_fwd(N, cu, H, DK, DV, q, k, v, beta, s0, o, pass ? ST : NULL, 2);
        rc |= dn_oracle_bwd(N, cu, H, DK, DV, q, k, v, beta, s0, d_o, dst, dq, dk, dv, db, pass ? dS0 : NULL, 2);
        rc |= dn_oracle_gated_fwd(N, cu, H, DK, DV, q, k, v, beta, g, s0, o, ST, 1);
        rc |= dn_oracle_gated_bwd(N, cu, H, DK, DV, q, k, v, beta, g, s0, d_o, dst, dq, dk, dv, db, dg, dS0, 1);
    }
    double sum = 0;
    for (size_t i = 0; i < T * H * DV; ++i) sum += o[i] + dv[i];
    for (size_t i = 0; i < T * H * DK; ++i) sum += dq[i] + dk[i];
    for (size_t i = 0; i < T * H; ++i) sum += db[i] + dg[i];
    for (size_t i = 0; i < st; ++i) sum += ST[i] + dS0[i];
    printf("oracle under sanitizers: rc=%d checksum=%.6f\n", rc, sum);
    free(q); free(k); free(v); free(beta); free(g); free(d_o); free(S0); free(dST);
    free(o); free(ST); free(dq); free(dk); free(dv); free(db); free(dg); free(dS0);
    return (rc != 0 || !isfinite(sum)) ? 1 : 0;
}
