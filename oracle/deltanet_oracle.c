/*
 * fp64 CPU oracle for the DeltaNet layer: the per-token delta-rule recurrence and its exact
 * reverse-mode gradient.  TEST INFRASTRUCTURE ONLY: nothing in the product path may call this.
 * It shares no code with the HIP path.
 *
 * What it computes (paper section 2.2, the delta update rule and the read-out; section 3.1,
 * the Householder form of the same update), per chain (sequence n, head h), with the state
 * stored in the orientation of the paper's pseudocode listing, S in R^{d_k x d_v}
 * (the transpose of the S in R^{d_v x d_k} of the running text):
 *
 *     S_0 = initial_state (or 0)
 *     for t = 1..len:
 *         e_t = v_t - S_{t-1}^T k_t            (target minus the value currently stored under k_t)
 *         S_t = S_{t-1} + beta_t k_t e_t^T     (== S_{t-1}(I - beta k k^T) + beta v k^T, transposed)
 *         o_t = S_t^T q_t                      (read-out from the UPDATED state)
 *     final_state = S_len
 *
 * No blocking, no chunking, no reordering: one token at a time, plain loops.
 *
 * The backward pass is not given by the paper (it only says states are recomputed); here it is
 * the exact adjoint of the loop above, taken token by token in reverse order.  With
 * G = dLoss/dS_t (starting from dfinal_state):
 *
 *     dq_t   = S_t do_t ;            G += q_t do_t^T
 *     g      = G^T k_t               (gradient w.r.t. the written vector beta_t e_t)
 *     dk_t   = beta_t G e_t - S_{t-1} (beta_t g)
 *     dbeta_t= g . e_t ;             dv_t = beta_t g
 *     G     -= k_t (beta_t g)^T      (now G = dLoss/dS_{t-1})
 *     dinitial_state = G after t = 1
 *
 * States needed in reverse order are rebuilt from checkpoints kept every SEG tokens.
 *
 * Layouts (all row-major, double): q,k [T,H,d_k]; v,o,do [T,H,d_v]; beta [T,H];
 * states [N,H,d_k,d_v]; cu_seqlens int32 [N+1] with cu[0]=0, cu[N]=T (a dense batch B x L is
 * N=B, cu[n]=n*L).  Threads (OpenMP) run over independent chains only.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SEG 64

static void step_forward(int dk, int dv, double *S, const double *k, const double *v, double beta,
                         double *e /* out, dv */)
{
    for (int j = 0; j < dv; ++j) {
        double acc = 0.0;
        for (int i = 0; i < dk; ++i) acc += S[(size_t)i * dv + j] * k[i];
        e[j] = v[j] - acc;
    }
    for (int i = 0; i < dk; ++i) {
        double bk = beta * k[i];
        for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] += bk * e[j];
    }
}

int dn_oracle_fwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k,
                  const double *v, const double *beta, const double *S0, double *o, double *ST,
                  int nthreads)
{
    if (N < 0 || H <= 0 || dk <= 0 || dv <= 0 || !cu) return -1;
    int nchains = N * H;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int c = 0; c < nchains; ++c) {
        int n = c / H, h = c % H;
        size_t sd = (size_t)dk * dv;
        double *S = (double *)malloc(sd * sizeof(double));
        double *e = (double *)malloc((size_t)dv * sizeof(double));
        if (!S || !e) { fail = 1; free(S); free(e); continue; }
        if (S0) memcpy(S, S0 + (size_t)c * sd, sd * sizeof(double));
        else memset(S, 0, sd * sizeof(double));
        for (int t = cu[n]; t < cu[n + 1]; ++t) {
            size_t row = (size_t)t * H + h;
            const double *qt = q + row * dk, *kt = k + row * dk, *vt = v + row * dv;
            step_forward(dk, dv, S, kt, vt, beta[row], e);
            double *ot = o + row * dv;
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(size_t)i * dv + j] * qt[i];
                ot[j] = acc;
            }
        }
        if (ST) memcpy(ST + (size_t)c * sd, S, sd * sizeof(double));
        free(S); free(e);
    }
    return fail ? -2 : 0;
}

int dn_oracle_bwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k,
                  const double *v, const double *beta, const double *S0, const double *d_o,
                  const double *dST, double *dq, double *dkk, double *dvv, double *dbeta, double *dS0,
                  int nthreads)
{
    if (N < 0 || H <= 0 || dk <= 0 || dv <= 0 || !cu) return -1;
    int nchains = N * H;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int c = 0; c < nchains; ++c) {
        int n = c / H, h = c % H;
        size_t sd = (size_t)dk * dv;
        int t0 = cu[n], len = cu[n + 1] - cu[n];
        int nseg = (len + SEG - 1) / SEG;
        /* ckpt[s] = state before the first token of segment s */
        double *ckpt = (double *)malloc((size_t)(nseg > 0 ? nseg : 1) * sd * sizeof(double));
        /* states[i] = state after i tokens of the current segment, i = 0..SEG */
        double *states = (double *)malloc((size_t)(SEG + 1) * sd * sizeof(double));
        double *es = (double *)malloc((size_t)SEG * dv * sizeof(double));
        double *G = (double *)malloc(sd * sizeof(double));
        double *g = (double *)malloc((size_t)dv * sizeof(double));
        if (!ckpt || !states || !es || !G || !g) {
            fail = 1; free(ckpt); free(states); free(es); free(G); free(g); continue;
        }
        /* forward sweep: checkpoints only */
        double *S = states;
        if (S0) memcpy(S, S0 + (size_t)c * sd, sd * sizeof(double));
        else memset(S, 0, sd * sizeof(double));
        for (int i = 0; i < len; ++i) {
            if (i % SEG == 0) memcpy(ckpt + (size_t)(i / SEG) * sd, S, sd * sizeof(double));
            size_t row = (size_t)(t0 + i) * H + h;
            step_forward(dk, dv, S, k + row * dk, v + row * dv, beta[row], es);
        }
        if (dST) memcpy(G, dST + (size_t)c * sd, sd * sizeof(double));
        else memset(G, 0, sd * sizeof(double));
        /* reverse sweep, one segment at a time */
        for (int s = nseg - 1; s >= 0; --s) {
            int i0 = s * SEG, i1 = i0 + SEG < len ? i0 + SEG : len;
            memcpy(states, ckpt + (size_t)s * sd, sd * sizeof(double));
            for (int i = i0; i < i1; ++i) {
                size_t row = (size_t)(t0 + i) * H + h;
                double *Sn = states + (size_t)(i - i0 + 1) * sd;
                memcpy(Sn, states + (size_t)(i - i0) * sd, sd * sizeof(double));
                step_forward(dk, dv, Sn, k + row * dk, v + row * dv, beta[row],
                             es + (size_t)(i - i0) * dv);
            }
            for (int i = i1 - 1; i >= i0; --i) {
                size_t row = (size_t)(t0 + i) * H + h;
                const double *qt = q + row * dk, *kt = k + row * dk, *dot = d_o + row * dv;
                const double *Sprev = states + (size_t)(i - i0) * sd;
                const double *Scur = states + (size_t)(i - i0 + 1) * sd;
                const double *e = es + (size_t)(i - i0) * dv;
                double b = beta[row];
                double *dqt = dq + row * dk, *dkt = dkk + row * dk, *dvt = dvv + row * dv;
                /* read-out o_t = S_t^T q_t */
                for (int a = 0; a < dk; ++a) {
                    double acc = 0.0;
                    for (int j = 0; j < dv; ++j) acc += Scur[(size_t)a * dv + j] * dot[j];
                    dqt[a] = acc;
                    for (int j = 0; j < dv; ++j) G[(size_t)a * dv + j] += qt[a] * dot[j];
                }
                /* write S_t = S_{t-1} + k (beta e)^T */
                for (int j = 0; j < dv; ++j) {
                    double acc = 0.0;
                    for (int a = 0; a < dk; ++a) acc += G[(size_t)a * dv + j] * kt[a];
                    g[j] = acc;
                }
                double db = 0.0;
                for (int j = 0; j < dv; ++j) { db += g[j] * e[j]; dvt[j] = b * g[j]; }
                dbeta[row] = db;
                for (int a = 0; a < dk; ++a) {
                    double acc = 0.0;
                    for (int j = 0; j < dv; ++j)
                        acc += G[(size_t)a * dv + j] * (b * e[j]) - Sprev[(size_t)a * dv + j] * (b * g[j]);
                    dkt[a] = acc;
                }
                /* e = v - S_{t-1}^T k feeds back into S_{t-1} */
                for (int a = 0; a < dk; ++a)
                    for (int j = 0; j < dv; ++j) G[(size_t)a * dv + j] -= kt[a] * (b * g[j]);
            }
        }
        if (dS0) memcpy(dS0 + (size_t)c * sd, G, sd * sizeof(double));
        free(ckpt); free(states); free(es); free(G); free(g);
    }
    return fail ? -2 : 0;
}

/*
 * Gated variant (the "Gated DeltaNet" row of the paper's overview table of linear recurrent models,
 * named in its limitations section as the remedy for length generalisation): a scalar decay
 * alpha_t = exp(g_t), g_t <= 0, multiplies the transition,
 *
 *     e_t = v_t - alpha_t S_{t-1}^T k_t
 *     S_t = alpha_t S_{t-1} + beta_t k_t e_t^T      (== S_{t-1} alpha_t (I - beta k k^T) + beta v k^T, transposed)
 *     o_t = S_t^T q_t
 *
 * and g = 0 gives back the plain recurrence above.  The paper prints no gradient; the reverse sweep
 * below is the exact adjoint of these three lines, with G = dLoss/dS_t:
 *
 *     dq_t = S_t do_t ;  G += q_t do_t^T
 *     w = G^T k_t ;  dbeta_t = w . e_t ;  de = beta_t w ;  dv_t = de
 *     dk_t = G (beta_t e_t) - alpha_t S_{t-1} de
 *     dalpha_t = <G, S_{t-1}> - de . (S_{t-1}^T k_t) ;  dg_t = alpha_t dalpha_t
 *     G <- alpha_t (G - k_t de^T)
 *
 * g and dg are [T,H] like beta.  Everything else as for the plain functions.
 */
#include <math.h>

static void step_forward_gated(int dk, int dv, double *S, const double *k, const double *v, double beta,
                               double alpha, double *e /* out, dv */)
{
    for (int j = 0; j < dv; ++j) {
        double acc = 0.0;
        for (int i = 0; i < dk; ++i) acc += S[(size_t)i * dv + j] * k[i];
        e[j] = v[j] - alpha * acc;
    }
    for (int i = 0; i < dk; ++i) {
        double bk = beta * k[i];
        for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] = alpha * S[(size_t)i * dv + j] + bk * e[j];
    }
}

int dn_oracle_gated_fwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k,
                        const double *v, const double *beta, const double *g, const double *S0, double *o,
                        double *ST, int nthreads)
{
    if (N < 0 || H <= 0 || dk <= 0 || dv <= 0 || !cu || !g) return -1;
    int nchains = N * H;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int c = 0; c < nchains; ++c) {
        int n = c / H, h = c % H;
        size_t sd = (size_t)dk * dv;
        double *S = (double *)malloc(sd * sizeof(double));
        double *e = (double *)malloc((size_t)dv * sizeof(double));
        if (!S || !e) { fail = 1; free(S); free(e); continue; }
        if (S0) memcpy(S, S0 + (size_t)c * sd, sd * sizeof(double));
        else memset(S, 0, sd * sizeof(double));
        for (int t = cu[n]; t < cu[n + 1]; ++t) {
            size_t row = (size_t)t * H + h;
            const double *qt = q + row * dk;
            step_forward_gated(dk, dv, S, k + row * dk, v + row * dv, beta[row], exp(g[row]), e);
            double *ot = o + row * dv;
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(size_t)i * dv + j] * qt[i];
                ot[j] = acc;
            }
        }
        if (ST) memcpy(ST + (size_t)c * sd, S, sd * sizeof(double));
        free(S); free(e);
    }
    return fail ? -2 : 0;
}

int dn_oracle_gated_bwd(int N, const int32_t *cu, int H, int dk, int dv, const double *q, const double *k,
                        const double *v, const double *beta, const double *g, const double *S0,
                        const double *d_o, const double *dST, double *dq, double *dkk, double *dvv,
                        double *dbeta, double *dg, double *dS0, int nthreads)
{
    if (N < 0 || H <= 0 || dk <= 0 || dv <= 0 || !cu || !g) return -1;
    int nchains = N * H;
    int fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int c = 0; c < nchains; ++c) {
        int n = c / H, h = c % H;
        size_t sd = (size_t)dk * dv;
        int t0 = cu[n], len = cu[n + 1] - cu[n];
        int nseg = (len + SEG - 1) / SEG;
        double *ckpt = (double *)malloc((size_t)(nseg > 0 ? nseg : 1) * sd * sizeof(double));
        double *states = (double *)malloc((size_t)(SEG + 1) * sd * sizeof(double));
        double *es = (double *)malloc((size_t)SEG * dv * sizeof(double));
        double *G = (double *)malloc(sd * sizeof(double));
        double *w = (double *)malloc((size_t)dv * sizeof(double));
        double *sk = (double *)malloc((size_t)dv * sizeof(double));
        if (!ckpt || !states || !es || !G || !w || !sk) {
            fail = 1; free(ckpt); free(states); free(es); free(G); free(w); free(sk); continue;
        }
        double *S = states;
        if (S0) memcpy(S, S0 + (size_t)c * sd, sd * sizeof(double));
        else memset(S, 0, sd * sizeof(double));
        for (int i = 0; i < len; ++i) { /* forward sweep: checkpoints only */
            if (i % SEG == 0) memcpy(ckpt + (size_t)(i / SEG) * sd, S, sd * sizeof(double));
            size_t row = (size_t)(t0 + i) * H + h;
            step_forward_gated(dk, dv, S, k + row * dk, v + row * dv, beta[row], exp(g[row]), es);
        }
        if (dST) memcpy(G, dST + (size_t)c * sd, sd * sizeof(double));
        else memset(G, 0, sd * sizeof(double));
        for (int s = nseg - 1; s >= 0; --s) {
            int i0 = s * SEG, i1 = i0 + SEG < len ? i0 + SEG : len;
            memcpy(states, ckpt + (size_t)s * sd, sd * sizeof(double));
            for (int i = i0; i < i1; ++i) {
                size_t row = (size_t)(t0 + i) * H + h;
                double *Sn = states + (size_t)(i - i0 + 1) * sd;
                memcpy(Sn, states + (size_t)(i - i0) * sd, sd * sizeof(double));
                step_forward_gated(dk, dv, Sn, k + row * dk, v + row * dv, beta[row], exp(g[row]),
                                   es + (size_t)(i - i0) * dv);
            }
            for (int i = i1 - 1; i >= i0; --i) {
                size_t row = (size_t)(t0 + i) * H + h;
                const double *qt = q + row * dk, *kt = k + row * dk, *dot = d_o + row * dv;
                const double *Sprev = states + (size_t)(i - i0) * sd;
                const double *Scur = states + (size_t)(i - i0 + 1) * sd;
                const double *e = es + (size_t)(i - i0) * dv;
                double b = beta[row], alpha = exp(g[row]);
                double *dqt = dq + row * dk, *dkt = dkk + row * dk, *dvt = dvv + row * dv;
                for (int a = 0; a < dk; ++a) { /* read-out */
                    double acc = 0.0;
                    for (int j = 0; j < dv; ++j) acc += Scur[(size_t)a * dv + j] * dot[j];
                    dqt[a] = acc;
                    for (int j = 0; j < dv; ++j) G[(size_t)a * dv + j] += qt[a] * dot[j];
                }
                for (int j = 0; j < dv; ++j) { /* w = G^T k, and S_{t-1}^T k */
                    double acc = 0.0, acc2 = 0.0;
                    for (int a = 0; a < dk; ++a) {
                        acc += G[(size_t)a * dv + j] * kt[a];
                        acc2 += Sprev[(size_t)a * dv + j] * kt[a];
                    }
                    w[j] = acc; sk[j] = acc2;
                }
                double db = 0.0, dalpha = 0.0;
                for (int j = 0; j < dv; ++j) { db += w[j] * e[j]; dvt[j] = b * w[j]; dalpha -= b * w[j] * sk[j]; }
                dbeta[row] = db;
                for (int a = 0; a < dk; ++a) {
                    double acc = 0.0;
                    for (int j = 0; j < dv; ++j) {
                        acc += G[(size_t)a * dv + j] * (b * e[j]) - alpha * Sprev[(size_t)a * dv + j] * (b * w[j]);
                        dalpha += G[(size_t)a * dv + j] * Sprev[(size_t)a * dv + j];
                    }
                    dkt[a] = acc;
                }
                dg[row] = alpha * dalpha;
                for (int a = 0; a < dk; ++a)
                    for (int j = 0; j < dv; ++j)
                        G[(size_t)a * dv + j] = alpha * (G[(size_t)a * dv + j] - kt[a] * (b * w[j]));
            }
        }
        if (dS0) memcpy(dS0 + (size_t)c * sd, G, sd * sizeof(double));
        free(ckpt); free(states); free(es); free(G); free(w); free(sk);
    }
    return fail ? -2 : 0;
}

int dn_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
