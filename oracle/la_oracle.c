/*
 * la_oracle.c: plain fp64 CPU oracle for kernelised linear attention with the
 * feature map phi(x) = elu(x) + 1 (paper eq. 7).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct checker
 * that the GPU library is compared against.  It shares no code, header, table
 * or helper with the HIP path, and nothing on the product path may call it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every function is a direct transcription of a definition or of the steps of
 * an algorithm in the paper, in the paper's order and notation, with no
 * blocking, fusion or reordering:
 *
 *   phi / dphi                       eq. 7 (elu with alpha = 1, plus one)
 *   causal_fwd_quadratic             eq. 8 with sim(q,k) = phi(q)^T phi(k)      (definition)
 *   causal_weights                   the row-normalised weights inside eq. 8    (definition)
 *   causal_fwd_prefix                eq. 10, 11, 12 (running sums S_i, Z_i)
 *   recurrent_step                   eq. 16-20 (s_i, z_i update, then read-out)
 *   global_fwd_quadratic             eq. 3 with the same sim                    (definition)
 *   global_fwd_linear                eq. 5 / eq. 6
 *   causal_numerator_fwd / _bwd      the numerator of eq. 9 and its gradients eq. 13-15
 *                                    (what Algorithm 1 computes), each as a cumulative
 *                                    sum of outer products applied per position
 *                                    (takes already-mapped phi(Q), phi(K))
 *   causal_bwd_quadratic             gradient of eq. 8 by brute force           (definition)
 *   global_bwd_quadratic             gradient of eq. 3 by brute force           (definition)
 *   global_bwd_linear                the same gradient from the two global sums
 *                                    sum_j phi(K_j)[V_j,1]^T and sum_i phi(Q_i) Gt_i^T
 *                                    (eq. 5-6 differentiated; no causal mask)
 *   causal_fwd_state                 eq. 10-12 started from a given (S_0, Z_0) instead of
 *                                    zero, also returning (S_N, Z_N): the RNN view of
 *                                    section 3.4 with its hidden state handed in and out
 *   causal_bwd_state                 backpropagation through time for that RNN: the
 *                                    loss gradient also arrives at (S_N, Z_N) and leaves
 *                                    at (S_0, Z_0); one sweep forward in time, one backward
 *   causal_bwd_linear                eq. 13-15 applied to values
 *                                    augmented with a column of ones, then the
 *                                    chain rule through phi (the paper leaves the
 *                                    denominator and the fraction to autograd,
 *                                    supplementary section A; this is that part
 *                                    written out)
 *
 * A switch (set_feature_map) replaces eq. 7 by the identity in all of the above:
 * Q and K are then taken as feature values of a map the caller applied.
 *
 * Readings of the paper that this file fixes (the paper is silent on each):
 *   - eps: den_i = phi(Q_i)^T Z_i + eps, added once after the dot product.
 *   - elu has alpha = 1; the branch is x > 0 (strict), so phi(0) = exp(0) = 1.
 *   - the causal sum is inclusive (j <= i); the recurrent step updates first,
 *     then reads.
 *   - gradients are with respect to the raw Q, K (through phi) and V.
 *
 * Layout: every tensor is row-major [BH, N, feature]; the BH slabs (one per
 * batch element and head) are independent problems.  OpenMP runs over slabs
 * only; inside a slab all sums run in ascending token order (descending for
 * the sums over j >= i).
 *
 * Pins (tests/test_oracle_*.py): prefix == quadratic == stepwise; linear
 * backward == brute-force backward == central finite differences == autograd
 * of the quadratic form; closed forms (Q = K = 0 gives a running mean, constant
 * V gives a constant output, N = 1); rational hand-worked case in tests/golden;
 * the state-carrying pair: a sequence cut in two and chained through the state
 * equals the uncut sequence (outputs and gradients), zero state equals the plain
 * functions, central finite differences with respect to S_0, Z_0.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Which feature map every function of this file applies to Q and K:           */
/*   0  eq. 7, phi(x) = elu(x) + 1 (the default);                                */
/*   1  the identity: Q and K already hold feature values phi(Q), phi(K) of some */
/*      other map (section 3.2 allows any non-negative one; Algorithm 1 itself   */
/*      is stated on already-mapped inputs), and gradients are with respect to   */
/*      those features.                                                          */
/* Set between calls, never during one.                                          */
static int g_feature_map = 0;
void la_oracle_set_feature_map(int which) { g_feature_map = which; }

/* eq. 7: phi(x) = elu(x) + 1 = x + 1 for x > 0, exp(x) otherwise. */
double la_oracle_phi(double x) {
    if (g_feature_map == 1) return x;
    return x > 0.0 ? x + 1.0 : exp(x);
}

/* derivative of eq. 7: 1 for x > 0, exp(x) otherwise. */
double la_oracle_dphi(double x) {
    if (g_feature_map == 1) return 1.0;
    return x > 0.0 ? 1.0 : exp(x);
}

int la_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void la_oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static double dot(const double *a, const double *b, int n) {
    double s = 0.0;
    for (int t = 0; t < n; ++t) s += a[t] * b[t];
    return s;
}

static double *map_rows(const double *X, long rows, int D, double (*f)(double)) {
    double *Y = (double *)malloc(sizeof(double) * (size_t)rows * (size_t)D);
    for (long t = 0; t < rows * D; ++t) Y[t] = f(X[t]);
    return Y;
}

/* ------------------------------------------------------------------------ */
/* eq. 8: V'_i = sum_{j<=i} sim(Q_i,K_j) V_j / sum_{j<=i} sim(Q_i,K_j),      */
/* sim(q,k) = phi(q)^T phi(k).  O(N^2).  den (may be NULL) gets the          */
/* denominator including eps.                                                */
void la_oracle_causal_fwd_quadratic(const double *Q, const double *K, const double *V,
                                    double *O, double *den,
                                    int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M;
        double *Os = O + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *num = (double *)malloc(sizeof(double) * (size_t)M);
        for (int i = 0; i < N; ++i) {
            double d = 0.0;
            for (int e = 0; e < M; ++e) num[e] = 0.0;
            for (int j = 0; j <= i; ++j) {
                double a = dot(fq + (size_t)i * D, fk + (size_t)j * D, D);
                for (int e = 0; e < M; ++e) num[e] += a * Vs[(size_t)j * M + e];
                d += a;
            }
            d += eps;
            for (int e = 0; e < M; ++e) Os[(size_t)i * M + e] = num[e] / d;
            if (den) den[(size_t)s * N + i] = d;
        }
        free(num); free(fq); free(fk);
    }
}

/* The normalised weights of eq. 8 for one slab: W[i][j] = sim(Q_i,K_j)/den_i  */
/* for j <= i, 0 for j > i.  W is [N, N].                                      */
void la_oracle_causal_weights(const double *Q, const double *K, double *W,
                              int N, int D, double eps) {
    double *fq = map_rows(Q, N, D, la_oracle_phi);
    double *fk = map_rows(K, N, D, la_oracle_phi);
    for (int i = 0; i < N; ++i) {
        double d = 0.0;
        for (int j = 0; j < N; ++j) {
            double a = j <= i ? dot(fq + (size_t)i * D, fk + (size_t)j * D, D) : 0.0;
            W[(size_t)i * N + j] = a;
            d += a;
        }
        d += eps;
        for (int j = 0; j < N; ++j) W[(size_t)i * N + j] /= d;
    }
    free(fq); free(fk);
}

/* ------------------------------------------------------------------------ */
/* eq. 16-20 for one token per slab: s <- s + phi(k) v^T, z <- z + phi(k),    */
/* out = phi(q)^T s / (phi(q)^T z + eps).  S is [BH, D, M], z is [BH, D].     */
void la_oracle_recurrent_step(const double *q, const double *k, const double *v,
                              double *S, double *z, double *out, double *den,
                              int BH, int D, int M, double eps) {
#pragma omp parallel for schedule(static)
    for (int s = 0; s < BH; ++s) {
        const double *qs = q + (size_t)s * D, *ks = k + (size_t)s * D, *vs = v + (size_t)s * M;
        double *Ss = S + (size_t)s * D * M, *zs = z + (size_t)s * D, *os = out + (size_t)s * M;
        for (int d = 0; d < D; ++d) {
            double fk = la_oracle_phi(ks[d]);
            for (int e = 0; e < M; ++e) Ss[(size_t)d * M + e] += fk * vs[e];   /* eq. 18 */
            zs[d] += fk;                                                        /* eq. 19 */
        }
        double dn = 0.0;
        for (int e = 0; e < M; ++e) os[e] = 0.0;
        for (int d = 0; d < D; ++d) {
            double fq = la_oracle_phi(qs[d]);
            for (int e = 0; e < M; ++e) os[e] += fq * Ss[(size_t)d * M + e];
            dn += fq * zs[d];
        }
        dn += eps;
        for (int e = 0; e < M; ++e) os[e] /= dn;                                /* eq. 20 */
        if (den) den[s] = dn;
    }
}

/* eq. 10-12: S_i = S_{i-1} + phi(K_i) V_i^T, Z_i = Z_{i-1} + phi(K_i),       */
/* V'_i = phi(Q_i)^T S_i / (phi(Q_i)^T Z_i + eps).  O(N D M).                 */
void la_oracle_causal_fwd_prefix(const double *Q, const double *K, const double *V,
                                 double *O, double *den,
                                 int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M;
        double *Os = O + (size_t)s * N * M;
        double *S = (double *)calloc((size_t)D * M, sizeof(double));
        double *Z = (double *)calloc((size_t)D, sizeof(double));
        double *fq = (double *)malloc(sizeof(double) * (size_t)D);
        for (int i = 0; i < N; ++i) {
            for (int d = 0; d < D; ++d) {
                double fk = la_oracle_phi(Ks[(size_t)i * D + d]);
                for (int e = 0; e < M; ++e) S[(size_t)d * M + e] += fk * Vs[(size_t)i * M + e];
                Z[d] += fk;
            }
            for (int d = 0; d < D; ++d) fq[d] = la_oracle_phi(Qs[(size_t)i * D + d]);
            double dn = dot(fq, Z, D) + eps;
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d) a += fq[d] * S[(size_t)d * M + e];
                Os[(size_t)i * M + e] = a / dn;
            }
            if (den) den[(size_t)s * N + i] = dn;
        }
        free(S); free(Z); free(fq);
    }
}

/* ------------------------------------------------------------------------ */
/* eq. 3 with sim = phi^T phi: every query attends to every key.  O(N^2).    */
void la_oracle_global_fwd_quadratic(const double *Q, const double *K, const double *V,
                                    double *O, int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M;
        double *Os = O + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *num = (double *)malloc(sizeof(double) * (size_t)M);
        for (int i = 0; i < N; ++i) {
            double d = 0.0;
            for (int e = 0; e < M; ++e) num[e] = 0.0;
            for (int j = 0; j < N; ++j) {
                double a = dot(fq + (size_t)i * D, fk + (size_t)j * D, D);
                for (int e = 0; e < M; ++e) num[e] += a * Vs[(size_t)j * M + e];
                d += a;
            }
            d += eps;
            for (int e = 0; e < M; ++e) Os[(size_t)i * M + e] = num[e] / d;
        }
        free(num); free(fq); free(fk);
    }
}

/* eq. 5-6: sum_j phi(K_j) V_j^T and sum_j phi(K_j) computed once, reused for */
/* every query.  O(N D M).                                                    */
void la_oracle_global_fwd_linear(const double *Q, const double *K, const double *V,
                                 double *O, int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M;
        double *Os = O + (size_t)s * N * M;
        double *S = (double *)calloc((size_t)D * M, sizeof(double));
        double *Z = (double *)calloc((size_t)D, sizeof(double));
        double *fq = (double *)malloc(sizeof(double) * (size_t)D);
        for (int j = 0; j < N; ++j)
            for (int d = 0; d < D; ++d) {
                double fk = la_oracle_phi(Ks[(size_t)j * D + d]);
                for (int e = 0; e < M; ++e) S[(size_t)d * M + e] += fk * Vs[(size_t)j * M + e];
                Z[d] += fk;
            }
        for (int i = 0; i < N; ++i) {
            for (int d = 0; d < D; ++d) fq[d] = la_oracle_phi(Qs[(size_t)i * D + d]);
            double dn = dot(fq, Z, D) + eps;
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d) a += fq[d] * S[(size_t)d * M + e];
                Os[(size_t)i * M + e] = a / dn;
            }
        }
        free(S); free(Z); free(fq);
    }
}

/* ------------------------------------------------------------------------ */
/* The numerator of eq. 9 and its three gradients (eq. 13, 14, 15) are all   */
/* of one form: a cumulative sum of outer products, applied at every         */
/* position to a vector of that position,                                     */
/*     T_i = sum over j on one side of i (i included) of a_j b_j^T  (C x M),  */
/*     out_i = T_i^T x_i  (length M)   or   out_i = T_i x_i  (length C).       */
/* This routine is that form and nothing else: it keeps the running T,       */
/* walks the positions upwards (j <= i) or downwards (j >= i), adds a_i b_i^T */
/* first (the sums are inclusive) and then applies T.  One slab.              */
enum { SUM_UP_TO_I = 0, SUM_FROM_I_ON = 1 };
enum { APPLY_T_TRANSPOSED = 0, APPLY_T = 1 };
static void cumulative_outer_apply(const double *a, const double *b, const double *x,
                                   double *out, int N, int C, int M, int side, int how) {
    double *T = (double *)calloc((size_t)C * M, sizeof(double));
    for (int step = 0; step < N; ++step) {
        const int i = side == SUM_UP_TO_I ? step : N - 1 - step;
        for (int d = 0; d < C; ++d)
            for (int e = 0; e < M; ++e)
                T[(size_t)d * M + e] += a[(size_t)i * C + d] * b[(size_t)i * M + e];
        if (how == APPLY_T_TRANSPOSED) {         /* x_i has C entries, out_i has M */
            for (int e = 0; e < M; ++e) {
                double acc = 0.0;
                for (int d = 0; d < C; ++d) acc += x[(size_t)i * C + d] * T[(size_t)d * M + e];
                out[(size_t)i * M + e] = acc;
            }
        } else {                                 /* x_i has M entries, out_i has C */
            for (int d = 0; d < C; ++d) {
                double acc = 0.0;
                for (int e = 0; e < M; ++e) acc += x[(size_t)i * M + e] * T[(size_t)d * M + e];
                out[(size_t)i * C + d] = acc;
            }
        }
    }
    free(T);
}

/* eq. 9, numerator: Vbar_i = (sum_{j<=i} phi(K_j) V_j^T)^T phi(Q_i).          */
/* Inputs are already mapped (fQ = phi(Q), fK = phi(K)); one slab.            */
static void numerator_fwd_slab(const double *fQ, const double *fK, const double *V,
                               double *Vbar, int N, int C, int M) {
    cumulative_outer_apply(fK, V, fQ, Vbar, N, C, M, SUM_UP_TO_I, APPLY_T_TRANSPOSED);
}

/* Its gradients for an upstream G = dL/dVbar:                               */
/*   eq. 13  grad phi(Q_i) = (sum_{j<=i} phi(K_j) V_j^T) G_i                  */
/*   eq. 14  grad phi(K_i) = (sum_{j>=i} phi(Q_j) G_j^T) V_i                  */
/*   eq. 15  grad V_i      = (sum_{j>=i} phi(Q_j) G_j^T)^T phi(K_i)           */
/* (each sum rebuilt by its own sweep: nothing is stored per position).      */
static void numerator_bwd_slab(const double *fQ, const double *fK, const double *V,
                               const double *G, double *gQ, double *gK, double *gV,
                               int N, int C, int M) {
    cumulative_outer_apply(fK, V, G, gQ, N, C, M, SUM_UP_TO_I, APPLY_T);
    cumulative_outer_apply(fQ, G, V, gK, N, C, M, SUM_FROM_I_ON, APPLY_T);
    cumulative_outer_apply(fQ, G, fK, gV, N, C, M, SUM_FROM_I_ON, APPLY_T_TRANSPOSED);
}

void la_oracle_causal_numerator_fwd(const double *fQ, const double *fK, const double *V,
                                    double *Vbar, int BH, int N, int C, int M) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s)
        numerator_fwd_slab(fQ + (size_t)s * N * C, fK + (size_t)s * N * C, V + (size_t)s * N * M,
                           Vbar + (size_t)s * N * M, N, C, M);
}

void la_oracle_causal_numerator_bwd(const double *fQ, const double *fK, const double *V,
                                    const double *G, double *gQ, double *gK, double *gV,
                                    int BH, int N, int C, int M) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s)
        numerator_bwd_slab(fQ + (size_t)s * N * C, fK + (size_t)s * N * C, V + (size_t)s * N * M,
                           G + (size_t)s * N * M, gQ + (size_t)s * N * C, gK + (size_t)s * N * C,
                           gV + (size_t)s * N * M, N, C, M);
}

/* ------------------------------------------------------------------------ */
/* Gradient of eq. 8 by brute force.  With A_ij = phi(Q_i)^T phi(K_j) (j<=i), */
/* den_i = sum_j A_ij + eps and O_i = sum_j A_ij V_j / den_i:                  */
/*   dL/dV_j  = sum_{i>=j} (A_ij/den_i) G_i                                    */
/*   dL/dA_ij = G_i^T (V_j - O_i) / den_i                                      */
/*   dL/dphi(Q_i) = sum_{j<=i} dL/dA_ij phi(K_j),                              */
/*   dL/dphi(K_j) = sum_{i>=j} dL/dA_ij phi(Q_i), then times phi'.             */
void la_oracle_causal_bwd_quadratic(const double *Q, const double *K, const double *V,
                                    const double *G, double *dQ, double *dK, double *dV,
                                    int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M, *Gs = G + (size_t)s * N * M;
        double *dQs = dQ + (size_t)s * N * D, *dKs = dK + (size_t)s * N * D;
        double *dVs = dV + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *A = (double *)malloc(sizeof(double) * (size_t)N);
        double *Oi = (double *)malloc(sizeof(double) * (size_t)M);
        memset(dQs, 0, sizeof(double) * (size_t)N * D);
        memset(dKs, 0, sizeof(double) * (size_t)N * D);
        memset(dVs, 0, sizeof(double) * (size_t)N * M);
        for (int i = 0; i < N; ++i) {
            double dn = 0.0;
            for (int e = 0; e < M; ++e) Oi[e] = 0.0;
            for (int j = 0; j <= i; ++j) {
                A[j] = dot(fq + (size_t)i * D, fk + (size_t)j * D, D);
                dn += A[j];
                for (int e = 0; e < M; ++e) Oi[e] += A[j] * Vs[(size_t)j * M + e];
            }
            dn += eps;
            for (int e = 0; e < M; ++e) Oi[e] /= dn;
            for (int j = 0; j <= i; ++j) {
                double dA = 0.0;
                for (int e = 0; e < M; ++e) {
                    dVs[(size_t)j * M + e] += (A[j] / dn) * Gs[(size_t)i * M + e];
                    dA += Gs[(size_t)i * M + e] * (Vs[(size_t)j * M + e] - Oi[e]);
                }
                dA /= dn;
                for (int d = 0; d < D; ++d) {
                    dQs[(size_t)i * D + d] += dA * fk[(size_t)j * D + d];
                    dKs[(size_t)j * D + d] += dA * fq[(size_t)i * D + d];
                }
            }
        }
        for (long t = 0; t < (long)N * D; ++t) {
            dQs[t] *= la_oracle_dphi(Qs[t]);
            dKs[t] *= la_oracle_dphi(Ks[t]);
        }
        free(A); free(Oi); free(fq); free(fk);
    }
}

/* Linear-time gradient.  Write the fraction as num_i / den_i with            */
/*   [num_i, den_i - eps] = phi(Q_i)^T sum_{j<=i} phi(K_j) [V_j, 1]^T,         */
/* i.e. the numerator of eq. 9 on values augmented with a ones column.        */
/* Its upstream gradient is Gt_i = [G_i / den_i, -(G_i . O_i) / den_i]         */
/* (quotient rule).  eq. 13-15 on (phi(Q), phi(K), [V,1], Gt) then              */
/* give the gradients for phi(Q), phi(K) and the augmented values; the ones   */
/* column's own gradient is dropped, and the chain rule through phi finishes. */
void la_oracle_causal_bwd_linear(const double *Q, const double *K, const double *V,
                                 const double *G, double *dQ, double *dK, double *dV,
                                 int BH, int N, int D, int M, double eps) {
    const int Ma = M + 1;
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M, *Gs = G + (size_t)s * N * M;
        double *dQs = dQ + (size_t)s * N * D, *dKs = dK + (size_t)s * N * D;
        double *dVs = dV + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *Va = (double *)malloc(sizeof(double) * (size_t)N * Ma);
        double *Nu = (double *)malloc(sizeof(double) * (size_t)N * Ma);
        double *Gt = (double *)malloc(sizeof(double) * (size_t)N * Ma);
        double *gVa = (double *)malloc(sizeof(double) * (size_t)N * Ma);
        for (int i = 0; i < N; ++i) {
            for (int e = 0; e < M; ++e) Va[(size_t)i * Ma + e] = Vs[(size_t)i * M + e];
            Va[(size_t)i * Ma + M] = 1.0;
        }
        numerator_fwd_slab(fq, fk, Va, Nu, N, D, Ma);
        for (int i = 0; i < N; ++i) {
            double dn = Nu[(size_t)i * Ma + M] + eps;
            double go = 0.0;
            for (int e = 0; e < M; ++e) {
                double o = Nu[(size_t)i * Ma + e] / dn;
                Gt[(size_t)i * Ma + e] = Gs[(size_t)i * M + e] / dn;
                go += Gs[(size_t)i * M + e] * o;
            }
            Gt[(size_t)i * Ma + M] = -go / dn;
        }
        numerator_bwd_slab(fq, fk, Va, Gt, dQs, dKs, gVa, N, D, Ma);
        for (int i = 0; i < N; ++i)
            for (int e = 0; e < M; ++e) dVs[(size_t)i * M + e] = gVa[(size_t)i * Ma + e];
        for (long t = 0; t < (long)N * D; ++t) {
            dQs[t] *= la_oracle_dphi(Qs[t]);
            dKs[t] *= la_oracle_dphi(Ks[t]);
        }
        free(fq); free(fk); free(Va); free(Nu); free(Gt); free(gVa);
    }
}

/* ------------------------------------------------------------------------ */
/* Gradient of eq. 3 (every query sees every key) by brute force: as        */
/* causal_bwd_quadratic with the sums over all j.                            */
void la_oracle_global_bwd_quadratic(const double *Q, const double *K, const double *V,
                                    const double *G, double *dQ, double *dK, double *dV,
                                    int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M, *Gs = G + (size_t)s * N * M;
        double *dQs = dQ + (size_t)s * N * D, *dKs = dK + (size_t)s * N * D;
        double *dVs = dV + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *A = (double *)malloc(sizeof(double) * (size_t)N);
        double *Oi = (double *)malloc(sizeof(double) * (size_t)M);
        memset(dQs, 0, sizeof(double) * (size_t)N * D);
        memset(dKs, 0, sizeof(double) * (size_t)N * D);
        memset(dVs, 0, sizeof(double) * (size_t)N * M);
        for (int i = 0; i < N; ++i) {
            double dn = 0.0;
            for (int e = 0; e < M; ++e) Oi[e] = 0.0;
            for (int j = 0; j < N; ++j) {
                A[j] = dot(fq + (size_t)i * D, fk + (size_t)j * D, D);
                dn += A[j];
                for (int e = 0; e < M; ++e) Oi[e] += A[j] * Vs[(size_t)j * M + e];
            }
            dn += eps;
            for (int e = 0; e < M; ++e) Oi[e] /= dn;
            for (int j = 0; j < N; ++j) {
                double dA = 0.0;
                for (int e = 0; e < M; ++e) {
                    dVs[(size_t)j * M + e] += (A[j] / dn) * Gs[(size_t)i * M + e];
                    dA += Gs[(size_t)i * M + e] * (Vs[(size_t)j * M + e] - Oi[e]);
                }
                dA /= dn;
                for (int d = 0; d < D; ++d) {
                    dQs[(size_t)i * D + d] += dA * fk[(size_t)j * D + d];
                    dKs[(size_t)j * D + d] += dA * fq[(size_t)i * D + d];
                }
            }
        }
        for (long t = 0; t < (long)N * D; ++t) {
            dQs[t] *= la_oracle_dphi(Qs[t]);
            dKs[t] *= la_oracle_dphi(Ks[t]);
        }
        free(A); free(Oi); free(fq); free(fk);
    }
}

/* Linear-time gradient of eq. 5-6.  With St = sum_j phi(K_j) [V_j, 1]^T       */
/* (D x (M+1)), [num_i, den_i - eps] = phi(Q_i)^T St and Gt_i as in the causal  */
/* case:  grad phi(Q_i) = St Gt_i;  Rt = sum_i phi(Q_i) Gt_i^T;                  */
/* grad phi(K_j) = Rt [V_j, 1];  grad V_j = (Rt^T phi(K_j))[0:M].                */
void la_oracle_global_bwd_linear(const double *Q, const double *K, const double *V,
                                 const double *G, double *dQ, double *dK, double *dV,
                                 int BH, int N, int D, int M, double eps) {
    const int Ma = M + 1;
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M, *Gs = G + (size_t)s * N * M;
        double *dQs = dQ + (size_t)s * N * D, *dKs = dK + (size_t)s * N * D;
        double *dVs = dV + (size_t)s * N * M;
        double *fq = map_rows(Qs, N, D, la_oracle_phi);
        double *fk = map_rows(Ks, N, D, la_oracle_phi);
        double *St = (double *)calloc((size_t)D * Ma, sizeof(double));
        double *Rt = (double *)calloc((size_t)D * Ma, sizeof(double));
        double *Gt = (double *)malloc(sizeof(double) * (size_t)Ma);
        for (int j = 0; j < N; ++j)
            for (int d = 0; d < D; ++d) {
                for (int e = 0; e < M; ++e)
                    St[(size_t)d * Ma + e] += fk[(size_t)j * D + d] * Vs[(size_t)j * M + e];
                St[(size_t)d * Ma + M] += fk[(size_t)j * D + d];
            }
        for (int i = 0; i < N; ++i) {
            double dn = eps;
            for (int d = 0; d < D; ++d) dn += fq[(size_t)i * D + d] * St[(size_t)d * Ma + M];
            double go = 0.0;
            for (int e = 0; e < M; ++e) {
                double num = 0.0;
                for (int d = 0; d < D; ++d) num += fq[(size_t)i * D + d] * St[(size_t)d * Ma + e];
                Gt[e] = Gs[(size_t)i * M + e] / dn;
                go += Gs[(size_t)i * M + e] * (num / dn);
            }
            Gt[M] = -go / dn;
            for (int d = 0; d < D; ++d) {
                double a = 0.0;
                for (int e = 0; e < Ma; ++e) {
                    a += St[(size_t)d * Ma + e] * Gt[e];
                    Rt[(size_t)d * Ma + e] += fq[(size_t)i * D + d] * Gt[e];
                }
                dQs[(size_t)i * D + d] = a * la_oracle_dphi(Qs[(size_t)i * D + d]);
            }
        }
        for (int j = 0; j < N; ++j) {
            for (int d = 0; d < D; ++d) {
                double a = Rt[(size_t)d * Ma + M];
                for (int e = 0; e < M; ++e) a += Rt[(size_t)d * Ma + e] * Vs[(size_t)j * M + e];
                dKs[(size_t)j * D + d] = a * la_oracle_dphi(Ks[(size_t)j * D + d]);
            }
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d) a += Rt[(size_t)d * Ma + e] * fk[(size_t)j * D + d];
                dVs[(size_t)j * M + e] = a;
            }
        }
        free(fq); free(fk); free(St); free(Rt); free(Gt);
    }
}

/* ------------------------------------------------------------------------ */
/* eq. 10-12 with the running sums started at (S0, Z0) [BH, D, M] / [BH, D]  */
/* (NULL: zero) and the sums after the last token returned in (S1, Z1)       */
/* (NULL: not wanted).  With zero initial state this is causal_fwd_prefix.   */
void la_oracle_causal_fwd_state(const double *Q, const double *K, const double *V,
                                const double *S0, const double *Z0, double *O, double *den,
                                double *S1, double *Z1,
                                int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M;
        double *Os = O + (size_t)s * N * M;
        double *S = (double *)calloc((size_t)D * M, sizeof(double));
        double *Z = (double *)calloc((size_t)D, sizeof(double));
        double *fq = (double *)malloc(sizeof(double) * (size_t)D);
        if (S0) memcpy(S, S0 + (size_t)s * D * M, sizeof(double) * (size_t)D * M);
        if (Z0) memcpy(Z, Z0 + (size_t)s * D, sizeof(double) * (size_t)D);
        for (int i = 0; i < N; ++i) {
            for (int d = 0; d < D; ++d) {
                double fk = la_oracle_phi(Ks[(size_t)i * D + d]);
                for (int e = 0; e < M; ++e) S[(size_t)d * M + e] += fk * Vs[(size_t)i * M + e];
                Z[d] += fk;
            }
            for (int d = 0; d < D; ++d) fq[d] = la_oracle_phi(Qs[(size_t)i * D + d]);
            double dn = dot(fq, Z, D) + eps;
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d) a += fq[d] * S[(size_t)d * M + e];
                Os[(size_t)i * M + e] = a / dn;
            }
            if (den) den[(size_t)s * N + i] = dn;
        }
        if (S1) memcpy(S1 + (size_t)s * D * M, S, sizeof(double) * (size_t)D * M);
        if (Z1) memcpy(Z1 + (size_t)s * D, Z, sizeof(double) * (size_t)D);
        free(S); free(Z); free(fq);
    }
}

/* Backpropagation through time for the recurrence above.  The loss reaches   */
/* the outputs through G_i = dL/dO_i and the final state through              */
/* dS1 = dL/dS_N, dZ1 = dL/dZ_N (NULL: zero).  Step i reads the state         */
/*   O_i = S_i^T phi(Q_i) / den_i,  den_i = phi(Q_i) . Z_i + eps,             */
/* so it sends into the state the gradient                                    */
/*   dS_i += phi(Q_i) (G_i/den_i)^T,   dZ_i += -(G_i . O_i)/den_i phi(Q_i),   */
/* and dL/dphi(Q_i) = S_i G_i/den_i - (G_i . O_i)/den_i Z_i.  The state       */
/* gradient then flows back through S_i = S_{i-1} + phi(K_i) V_i^T,           */
/* Z_i = Z_{i-1} + phi(K_i):  dL/dphi(K_i) = dS_i V_i + dZ_i,                 */
/* dL/dV_i = dS_i^T phi(K_i), and dS_{i-1} = dS_i, dZ_{i-1} = dZ_i.  What is   */
/* left after token 1 is dL/dS_0, dL/dZ_0 (returned in dS0, dZ0 unless NULL).  */
/* A first loop runs forward to get S_i (for dQ), a second one backward.      */
void la_oracle_causal_bwd_state(const double *Q, const double *K, const double *V,
                                const double *S0, const double *Z0, const double *G,
                                const double *dS1, const double *dZ1,
                                double *dQ, double *dK, double *dV, double *dS0, double *dZ0,
                                int BH, int N, int D, int M, double eps) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < BH; ++s) {
        const double *Qs = Q + (size_t)s * N * D, *Ks = K + (size_t)s * N * D;
        const double *Vs = V + (size_t)s * N * M, *Gs = G + (size_t)s * N * M;
        double *dQs = dQ + (size_t)s * N * D, *dKs = dK + (size_t)s * N * D;
        double *dVs = dV + (size_t)s * N * M;
        double *S = (double *)calloc((size_t)D * M, sizeof(double));
        double *Z = (double *)calloc((size_t)D, sizeof(double));
        double *gS = (double *)calloc((size_t)D * M, sizeof(double));
        double *gZ = (double *)calloc((size_t)D, sizeof(double));
        double *fq = (double *)malloc(sizeof(double) * (size_t)D);
        double *Gb = (double *)malloc(sizeof(double) * (size_t)N * M);   /* G_i / den_i      */
        double *dl = (double *)malloc(sizeof(double) * (size_t)N);       /* -(G_i.O_i)/den_i */
        if (S0) memcpy(S, S0 + (size_t)s * D * M, sizeof(double) * (size_t)D * M);
        if (Z0) memcpy(Z, Z0 + (size_t)s * D, sizeof(double) * (size_t)D);
        if (dS1) memcpy(gS, dS1 + (size_t)s * D * M, sizeof(double) * (size_t)D * M);
        if (dZ1) memcpy(gZ, dZ1 + (size_t)s * D, sizeof(double) * (size_t)D);
        /* forward in time: the state, the outputs, and the gradient for phi(Q) */
        for (int i = 0; i < N; ++i) {
            for (int d = 0; d < D; ++d) {
                double fk = la_oracle_phi(Ks[(size_t)i * D + d]);
                for (int e = 0; e < M; ++e) S[(size_t)d * M + e] += fk * Vs[(size_t)i * M + e];
                Z[d] += fk;
            }
            for (int d = 0; d < D; ++d) fq[d] = la_oracle_phi(Qs[(size_t)i * D + d]);
            double dn = dot(fq, Z, D) + eps;
            double go = 0.0;
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d) a += fq[d] * S[(size_t)d * M + e];
                go += Gs[(size_t)i * M + e] * (a / dn);
                Gb[(size_t)i * M + e] = Gs[(size_t)i * M + e] / dn;
            }
            dl[i] = -go / dn;
            for (int d = 0; d < D; ++d) {
                double a = dl[i] * Z[d];
                for (int e = 0; e < M; ++e) a += S[(size_t)d * M + e] * Gb[(size_t)i * M + e];
                dQs[(size_t)i * D + d] = a * la_oracle_dphi(Qs[(size_t)i * D + d]);
            }
        }
        /* backward in time: the state gradient, and the gradients for phi(K) and V */
        for (int i = N - 1; i >= 0; --i) {
            for (int d = 0; d < D; ++d) {
                double q = la_oracle_phi(Qs[(size_t)i * D + d]);
                for (int e = 0; e < M; ++e) gS[(size_t)d * M + e] += q * Gb[(size_t)i * M + e];
                gZ[d] += dl[i] * q;
            }
            for (int d = 0; d < D; ++d) {
                double a = gZ[d];
                for (int e = 0; e < M; ++e) a += gS[(size_t)d * M + e] * Vs[(size_t)i * M + e];
                dKs[(size_t)i * D + d] = a * la_oracle_dphi(Ks[(size_t)i * D + d]);
            }
            for (int e = 0; e < M; ++e) {
                double a = 0.0;
                for (int d = 0; d < D; ++d)
                    a += gS[(size_t)d * M + e] * la_oracle_phi(Ks[(size_t)i * D + d]);
                dVs[(size_t)i * M + e] = a;
            }
        }
        if (dS0) memcpy(dS0 + (size_t)s * D * M, gS, sizeof(double) * (size_t)D * M);
        if (dZ0) memcpy(dZ0 + (size_t)s * D, gZ, sizeof(double) * (size_t)D);
        free(S); free(Z); free(gS); free(gZ); free(fq); free(Gb); free(dl);
    }
}
