/*
 * fp64 CPU oracle for the low-rank delta-rule recurrence of ParallelFlow (arXiv 2504.00492).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  It shares no code with the HIP path and must never be called from it.
 *
 * What it computes (one head; heads are independent):
 *
 *   general form   S_{t+1} = S_t + S_t A_t B_t^T + Atil_t B_t^T          (Section 3.1, the
 *                  discretised dynamics that follow the piecewise-linear driver equation)
 *                  o_t     = S_{t+1} q_t                                  (Section 1.1, "memory
 *                  readout": the state that already contains token t)
 *
 *   with S in R^{d_v x d_k}, A_t, B_t in R^{d_k x R}, Atil_t in R^{d_v x R}.  All R columns of a
 *   token act on the same old state: A_t B_t^T is ONE rank-R increment (Section 3.1, driver
 *   parameterisation), not a product of R rank-1 factors.
 *
 *   delta form     A_t = [beta_j k_j]_j,  Atil_t = [-beta_j v_j]_j,  B_t = [-k_j]_j
 *                  (Remark after the discretisation scheme, extended column by column to rank R),
 *                  which for R = 1 is the DeltaNet update of Section 1.3:
 *                  S_t = S_{t-1} - beta_t S_{t-1} k_t k_t^T + beta_t v_t k_t^T.
 *
 * Storage is "row form" (Remark after Theorem 3.2): A[t][j][:] is column j of A_t.
 * No blocking, no chunking, no reordering: token by token, column by column.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One head, general drivers.
 *   A    [L][R][dk]   Atil [L][R][dv]   Bm [L][R][dk]   Q [L][dk]
 *   S0   [dv][dk] (may be NULL = zeros)   O [L][dv] (may be NULL)   SL [dv][dk] (may be NULL)
 * Returns 0, or -1 if scratch memory could not be obtained. */
int pf_oracle_flow_head(const double *A, const double *Atil, const double *Bm, const double *Q,
                        const double *S0, double *O, double *SL,
                        int L, int R, int dk, int dv)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)dv * dk);
    double *c = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1) * dv);
    if (!S || !c) { free(S); free(c); return -1; }
    if (S0) memcpy(S, S0, sizeof(double) * (size_t)dv * dk);
    else    memset(S, 0, sizeof(double) * (size_t)dv * dk);

    for (int t = 0; t < L; ++t) {
        /* c_j = S a_j + atil_j  for every column j, all from the OLD state */
        for (int j = 0; j < R; ++j) {
            const double *a  = A    + ((size_t)t * R + j) * dk;
            const double *at = Atil + ((size_t)t * R + j) * dv;
            for (int m = 0; m < dv; ++m) {
                double acc = 0.0;
                for (int x = 0; x < dk; ++x) acc += S[(size_t)m * dk + x] * a[x];
                c[(size_t)j * dv + m] = acc + at[m];
            }
        }
        /* S <- S + sum_j c_j b_j^T */
        for (int j = 0; j < R; ++j) {
            const double *b = Bm + ((size_t)t * R + j) * dk;
            for (int m = 0; m < dv; ++m) {
                const double cm = c[(size_t)j * dv + m];
                for (int x = 0; x < dk; ++x) S[(size_t)m * dk + x] += cm * b[x];
            }
        }
        /* o_t = S q_t with the updated state */
        if (O) {
            const double *q = Q + (size_t)t * dk;
            for (int m = 0; m < dv; ++m) {
                double acc = 0.0;
                for (int x = 0; x < dk; ++x) acc += S[(size_t)m * dk + x] * q[x];
                O[(size_t)t * dv + m] = acc;
            }
        }
    }
    if (SL) memcpy(SL, S, sizeof(double) * (size_t)dv * dk);
    free(S); free(c);
    return 0;
}

/* Batched delta form over N independent heads, float inputs widened to double.
 *   Q [N][L][dk]  K [N][L][R][dk]  V [N][L][R][dv]  beta [N][L][R]  S0 [N][dv][dk] or NULL
 *   O [N][L][dv] or NULL            SL [N][dv][dk] or NULL
 * The delta mapping is applied literally (A = beta k, Atil = -beta v, B = -k) and the general
 * routine above does the work.  nthreads <= 0 means "whatever OpenMP picks".
 * Returns 0 on success, -1 on allocation failure. */
int pf_oracle_delta_fwd(const float *Q, const float *K, const float *V, const float *beta,
                        const float *S0, double *O, double *SL,
                        int N, int L, int R, int dk, int dv, int nthreads)
{
    int status = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < N; ++h) {
        const size_t nk = (size_t)L * R * dk, nv = (size_t)L * R * dv, nq = (size_t)L * dk;
        double *A  = (double *)malloc(sizeof(double) * (nk ? nk : 1));
        double *Bm = (double *)malloc(sizeof(double) * (nk ? nk : 1));
        double *At = (double *)malloc(sizeof(double) * (nv ? nv : 1));
        double *Qd = (double *)malloc(sizeof(double) * (nq ? nq : 1));
        double *S0d = (double *)malloc(sizeof(double) * (size_t)dv * dk);
        if (!A || !Bm || !At || !Qd || !S0d) {
#pragma omp atomic write
            status = -1;
        } else {
            const float *k = K + (size_t)h * nk, *v = V + (size_t)h * nv;
            const float *b = beta + (size_t)h * L * R, *q = Q + (size_t)h * nq;
            for (size_t tj = 0; tj < (size_t)L * R; ++tj) {
                const double bt = (double)b[tj];
                for (int x = 0; x < dk; ++x) {
                    A [tj * dk + x] =  bt * (double)k[tj * dk + x];
                    Bm[tj * dk + x] = -(double)k[tj * dk + x];
                }
                for (int m = 0; m < dv; ++m) At[tj * dv + m] = -bt * (double)v[tj * dv + m];
            }
            for (size_t i = 0; i < nq; ++i) Qd[i] = (double)q[i];
            for (size_t i = 0; i < (size_t)dv * dk; ++i)
                S0d[i] = S0 ? (double)S0[(size_t)h * dv * dk + i] : 0.0;
            int rc = pf_oracle_flow_head(A, At, Bm, Qd, S0d,
                                         O ? O + (size_t)h * L * dv : NULL,
                                         SL ? SL + (size_t)h * dv * dk : NULL, L, R, dk, dv);
            if (rc != 0) {
#pragma omp atomic write
                status = -1;
            }
        }
        free(A); free(Bm); free(At); free(Qd); free(S0d);
    }
    return status;
}

/* The same batched delta form, held against a candidate result instead of being returned: for
 * every head the recurrence above is run as it stands, and the candidate's O (float, [N][L][dv])
 * and final state (float, [N][dv][dk], may be NULL) are compared with it token by token.  Only
 * sums come back, so every head of a full-size workload can be checked without keeping the
 * fp64 outputs of all of them:
 *   err2 [N][L]   |o_t(candidate) - o_t|^2        ref2 [N][L]   |o_t|^2
 *   maxabs [N]    max over (t, m) of |o_t(candidate)[m] - o_t[m]|
 *   s_err2 [N], s_ref2 [N]   the same two sums over the final state (untouched if SLc is NULL)
 * No arithmetic of the method lives here: pf_oracle_flow_head produces the reference.
 * Returns 0 on success, -1 on allocation failure. */
int pf_oracle_delta_compare(const float *Q, const float *K, const float *V, const float *beta,
                            const float *S0, const float *Oc, const float *SLc,
                            double *err2, double *ref2, double *maxabs, double *s_err2, double *s_ref2,
                            int N, int L, int R, int dk, int dv, int nthreads)
{
    int status = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < N; ++h) {
        const size_t no = (size_t)L * dv, ns = (size_t)dv * dk;
        double *O  = (double *)malloc(sizeof(double) * (no ? no : 1));
        double *SL = (double *)malloc(sizeof(double) * ns);
        int rc = (O && SL) ? 0 : -1;
        if (rc == 0)
            rc = pf_oracle_delta_fwd(Q + (size_t)h * L * dk, K + (size_t)h * L * R * dk, V + (size_t)h * L * R * dv,
                                     beta + (size_t)h * L * R, S0 ? S0 + h * ns : NULL, O, SL, 1, L, R, dk, dv, -1);
        if (rc != 0) {
#pragma omp atomic write
            status = -1;
        } else {
            double worst = 0.0;
            for (int t = 0; t < L; ++t) {
                double e2 = 0.0, r2 = 0.0;
                for (int m = 0; m < dv; ++m) {
                    const double ref = O[(size_t)t * dv + m];
                    const double dif = (double)Oc[(size_t)h * no + (size_t)t * dv + m] - ref;
                    e2 += dif * dif;
                    r2 += ref * ref;
                    if (dif > worst) worst = dif;
                    if (-dif > worst) worst = -dif;
                }
                err2[(size_t)h * L + t] = e2;
                ref2[(size_t)h * L + t] = r2;
            }
            maxabs[h] = worst;
            if (SLc) {
                double e2 = 0.0, r2 = 0.0;
                for (size_t i = 0; i < ns; ++i) {
                    const double dif = (double)SLc[h * ns + i] - SL[i];
                    e2 += dif * dif;
                    r2 += SL[i] * SL[i];
                }
                s_err2[h] = e2;
                s_ref2[h] = r2;
            }
        }
        free(O); free(SL);
    }
    return status;
}

int pf_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
