/*
 * CPU oracle for the per-layer K-FAC second-order update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  It shares no code with the library and the
 * library never calls it.  Everything is written as the textbook definition in
 * double precision: nested loops, no blocking, no BLAS/LAPACK.  The only
 * concession to run time is an OpenMP "parallel for" over independent output
 * rows.
 *
 * What each function follows (DP-KFAC paper, arXiv 2206.15143):
 *   oracle_patches            - conv layer seen as a linear map over im2col
 *                               patches (footnote of section 3); bias handled by
 *                               a homogeneous 1 appended as the last column.
 *   oracle_rows_from_nchw     - rows (n, oh, ow) of a NCHW tensor, i.e. the
 *                               per-position vectors g whose second moment is G.
 *   oracle_factor             - Kronecker factors of Eq. 4 (section 2.2):
 *                               F = scale * sum_r x_r x_r^T.
 *   oracle_running_average    - Eqs. 10-11 (section 4.1) with `decay` the
 *                               weight on the old running factor.
 *   oracle_inverse_gj         - (M + damping I)^{-1} of section 5.2 by
 *                               Gauss-Jordan elimination with partial pivoting.
 *   oracle_pi_damping         - the two damping terms of the factored Tikhonov split (Eq. 12):
 *                               pi = sqrt((tr A / dim A) / (tr G / dim G)),
 *                               lambda_A = pi sqrt(gamma), lambda_G = sqrt(gamma) / pi
 *   oracle_inverse_chol       - same result through Cholesky (the technique
 *                               section 5.2 names); used to cross-check the
 *                               Gauss-Jordan route.
 *   oracle_precondition       - right-hand side of Eq. 12 / Eq. 5:
 *                               P = G_inv * grad * A_inv.
 *   oracle_eigh_jacobi        - eigen-decomposition M = Q diag(v) Q^T of a symmetric factor
 *                               (the Q_A, v_A, Q_G, v_G of Eq. 13) by the classical cyclic
 *                               Jacobi rotation method; eigenvalues ascending.
 *   oracle_precondition_eigen - Eq. 13 given eigen-decompositions.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, brute-force
 * Kronecker product, Woodbury identity, direct convolution, rank, PSD).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* x: NCHW [B, C, H, W] (float bits as given to the GPU).  out: row-major
 * [B*Ho*Wo, C*kh*kw (+1)]; row (n, oh, ow), column (c, i, j); zero padding of
 * pad_h rows above and below and pad_w columns left and right of the map;
 * last column is 1 when has_bias. */
void oracle_patches(const float *x, int B, int C, int H, int W, int kh, int kw, int stride, int pad_h, int pad_w,
                    int has_bias, double *out)
{
    const int Ho = (H + 2 * pad_h - kh) / stride + 1;
    const int Wo = (W + 2 * pad_w - kw) / stride + 1;
    const long dA = (long)C * kh * kw + (has_bias ? 1 : 0);
#pragma omp parallel for schedule(static)
    for (long nr = 0; nr < (long)B * Ho; ++nr) {
        const int n = (int)(nr / Ho), oh = (int)(nr % Ho);
        for (int ow = 0; ow < Wo; ++ow) {
            double *row = out + (((long)n * Ho + oh) * Wo + ow) * dA;
            for (int c = 0; c < C; ++c)
                for (int i = 0; i < kh; ++i)
                    for (int j = 0; j < kw; ++j) {
                        const int ih = oh * stride - pad_h + i;
                        const int iw = ow * stride - pad_w + j;
                        double v = 0.0;
                        if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                            v = (double)x[(((long)n * C + c) * H + ih) * W + iw];
                        row[((long)c * kh + i) * kw + j] = v;
                    }
            if (has_bias) row[dA - 1] = 1.0;
        }
    }
}

/* rows [R, d_in] (+1 homogeneous column) for a linear layer */
void oracle_linear_rows(const float *a, long R, int d_in, int has_bias, double *out)
{
    const long dA = d_in + (has_bias ? 1 : 0);
    for (long r = 0; r < R; ++r) {
        for (int u = 0; u < d_in; ++u) out[r * dA + u] = (double)a[r * d_in + u];
        if (has_bias) out[r * dA + d_in] = 1.0;
    }
}

/* g: NCHW [B, C, H, W] -> out [B*H*W, C], row (n, h, w) */
void oracle_rows_from_nchw(const float *g, int B, int C, int H, int W, double *out)
{
    for (int n = 0; n < B; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    out[(((long)n * H + h) * W + w) * C + c] = (double)g[(((long)n * C + c) * H + h) * W + w];
}

/* F[u][v] = scale * sum_r X[r][u] * X[r][v], full d x d */
void oracle_factor(const double *X, long R, int d, double scale, double *F)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < d; ++u) {
        double *Fu = F + (long)u * d;
        for (int v = 0; v < d; ++v) Fu[v] = 0.0;
        for (long r = 0; r < R; ++r) {
            const double xu = X[r * d + u];
            const double *Xr = X + r * d;
            for (int v = 0; v < d; ++v) Fu[v] += xu * Xr[v];
        }
        for (int v = 0; v < d; ++v) Fu[v] *= scale;
    }
}

/* single entry F[u][v] of the same definition, straight from the rows (used
 * to sample entries of very large factors) */
double oracle_factor_entry(const double *X, long R, int d, double scale, int u, int v)
{
    double s = 0.0;
    for (long r = 0; r < R; ++r) s += X[r * d + u] * X[r * d + v];
    return s * scale;
}

/* F_run <- decay * F_run + (1 - decay) * F_new */
void oracle_running_average(double *F_run, const double *F_new, int d, double decay)
{
    for (long i = 0; i < (long)d * d; ++i) F_run[i] = decay * F_run[i] + (1.0 - decay) * F_new[i];
}

/* Minv = (M + damping I)^{-1}; Gauss-Jordan on [M | I] with partial pivoting.
 * Returns 0, or k+1 if no usable pivot is found in column k. */
int oracle_inverse_gj(const double *M, int n, double damping, double *Minv)
{
    double *W = (double *)malloc(sizeof(double) * (size_t)n * n);
    if (!W) return -1;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            W[(long)i * n + j] = M[(long)i * n + j] + (i == j ? damping : 0.0);
            Minv[(long)i * n + j] = (i == j) ? 1.0 : 0.0;
        }
    for (int k = 0; k < n; ++k) {
        int p = k;
        double best = fabs(W[(long)k * n + k]);
        for (int i = k + 1; i < n; ++i)
            if (fabs(W[(long)i * n + k]) > best) { best = fabs(W[(long)i * n + k]); p = i; }
        if (!(best > 0.0)) { free(W); return k + 1; }
        if (p != k)
            for (int j = 0; j < n; ++j) {
                double t = W[(long)k * n + j]; W[(long)k * n + j] = W[(long)p * n + j]; W[(long)p * n + j] = t;
                t = Minv[(long)k * n + j]; Minv[(long)k * n + j] = Minv[(long)p * n + j]; Minv[(long)p * n + j] = t;
            }
        const double inv = 1.0 / W[(long)k * n + k];
        for (int j = 0; j < n; ++j) { W[(long)k * n + j] *= inv; Minv[(long)k * n + j] *= inv; }
#pragma omp parallel for schedule(static)
        for (int i = 0; i < n; ++i) {
            if (i == k) continue;
            const double f = W[(long)i * n + k];
            if (f == 0.0) continue;
            for (int j = 0; j < n; ++j) {
                W[(long)i * n + j] -= f * W[(long)k * n + j];
                Minv[(long)i * n + j] -= f * Minv[(long)k * n + j];
            }
        }
    }
    free(W);
    return 0;
}

/* Same inverse through M + damping I = L L^T, X = L^{-1}, Minv = X^T X.
 * Returns 0, or k+1 if pivot k is not positive (matrix not SPD). */
int oracle_inverse_chol(const double *M, int n, double damping, double *Minv)
{
    double *L = (double *)calloc((size_t)n * n, sizeof(double));
    double *X = (double *)calloc((size_t)n * n, sizeof(double));
    if (!L || !X) { free(L); free(X); return -1; }
    for (int j = 0; j < n; ++j) {
        double d = M[(long)j * n + j] + damping;
        for (int k = 0; k < j; ++k) d -= L[(long)j * n + k] * L[(long)j * n + k];
        if (!(d > 0.0)) { free(L); free(X); return j + 1; }
        L[(long)j * n + j] = sqrt(d);
        for (int i = j + 1; i < n; ++i) {
            double s = M[(long)i * n + j];
            for (int k = 0; k < j; ++k) s -= L[(long)i * n + k] * L[(long)j * n + k];
            L[(long)i * n + j] = s / L[(long)j * n + j];
        }
    }
    /* X = L^{-1} by forward substitution, column by column */
    for (int c = 0; c < n; ++c)
        for (int i = c; i < n; ++i) {
            double s = (i == c) ? 1.0 : 0.0;
            for (int k = c; k < i; ++k) s -= L[(long)i * n + k] * X[(long)k * n + c];
            X[(long)i * n + c] = s / L[(long)i * n + i];
        }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            const int k0 = i > j ? i : j;
            for (int k = k0; k < n; ++k) s += X[(long)k * n + i] * X[(long)k * n + j];
            Minv[(long)i * n + j] = s;
        }
    free(L); free(X);
    return 0;
}

/* Eq. 12: (A (x) G + gamma I)^-1 is approximated by (A + pi sqrt(gamma) I)^-1 (x) (G + sqrt(gamma)/pi I)^-1
 * with pi^2 = (tr A / dim A) / (tr G / dim G).  out[0] = lambda_A, out[1] = lambda_G.  A trace that is
 * not positive leaves pi = 1 (the split is then the symmetric one). */
void oracle_pi_damping(const double *A, int dA, const double *G, int dG, double gamma, double *out)
{
    double trA = 0.0, trG = 0.0;
    for (int i = 0; i < dA; ++i) trA += A[(long)i * dA + i];
    for (int i = 0; i < dG; ++i) trG += G[(long)i * dG + i];
    double pi = 1.0;
    if (trA > 0.0 && trG > 0.0) pi = sqrt((trA / dA) / (trG / dG));
    out[0] = pi * sqrt(gamma);
    out[1] = sqrt(gamma) / pi;
}

/* Eq. 5 / right-hand side of Eq. 12: P = Ginv [dG x dG] * grad [dG x dA] * Ainv [dA x dA] */
void oracle_precondition(const double *Ginv, const double *grad, const double *Ainv, int dG, int dA, double *P)
{
    double *T = (double *)malloc(sizeof(double) * (size_t)dG * dA);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dG; ++k) s += Ginv[(long)i * dG + k] * grad[(long)k * dA + j];
            T[(long)i * dA + j] = s;
        }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < dG; ++i)
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dA; ++k) s += T[(long)i * dA + k] * Ainv[(long)k * dA + j];
            P[(long)i * dA + j] = s;
        }
    free(T);
}

/* Symmetric eigen-decomposition by cyclic Jacobi: sweep over all (p, q), p < q, and annihilate M[p][q] by the
 * plane rotation whose tangent is the smaller root of t^2 + 2 tau t - 1 = 0, tau = (M[q][q] - M[p][p]) / (2 M[p][q]);
 * the product of the rotations is Q.  Stops when the off-diagonal norm is below 1e-15 of the total norm
 * (or after 60 sweeps).  On exit v is ascending and column k of Q (row-major n x n) belongs to v[k].
 * Returns the number of sweeps. */
int oracle_eigh_jacobi(const double *M, int n, double *Q, double *v)
{
    double *A = (double *)malloc(sizeof(double) * (size_t)n * n);
    memcpy(A, M, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) Q[(long)i * n + j] = (i == j) ? 1.0 : 0.0;
    int sweep = 0;
    for (; sweep < 60; ++sweep) {
        double off = 0.0, tot = 0.0;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                const double a = A[(long)i * n + j];
                tot += a * a;
                if (i != j) off += a * a;
            }
        if (off <= 1e-30 * tot) break;
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                const double apq = A[(long)p * n + q];
                if (apq == 0.0) continue;
                const double tau = (A[(long)q * n + q] - A[(long)p * n + p]) / (2.0 * apq);
                const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
                const double c = 1.0 / sqrt(1.0 + t * t), sn = t * c;
                for (int k = 0; k < n; ++k) {          /* columns p, q:  A <- A J */
                    const double akp = A[(long)k * n + p], akq = A[(long)k * n + q];
                    A[(long)k * n + p] = c * akp - sn * akq;
                    A[(long)k * n + q] = sn * akp + c * akq;
                }
                for (int k = 0; k < n; ++k) {          /* rows p, q:  A <- J^T A */
                    const double apk = A[(long)p * n + k], aqk = A[(long)q * n + k];
                    A[(long)p * n + k] = c * apk - sn * aqk;
                    A[(long)q * n + k] = sn * apk + c * aqk;
                }
                for (int k = 0; k < n; ++k) {          /* Q <- Q J */
                    const double qkp = Q[(long)k * n + p], qkq = Q[(long)k * n + q];
                    Q[(long)k * n + p] = c * qkp - sn * qkq;
                    Q[(long)k * n + q] = sn * qkp + c * qkq;
                }
            }
    }
    for (int i = 0; i < n; ++i) v[i] = A[(long)i * n + i];
    /* ascending order (selection sort, columns of Q follow) */
    for (int i = 0; i < n - 1; ++i) {
        int m = i;
        for (int j = i + 1; j < n; ++j)
            if (v[j] < v[m]) m = j;
        if (m != i) {
            const double tv = v[i]; v[i] = v[m]; v[m] = tv;
            for (int k = 0; k < n; ++k) {
                const double tq = Q[(long)k * n + i];
                Q[(long)k * n + i] = Q[(long)k * n + m];
                Q[(long)k * n + m] = tq;
            }
        }
    }
    free(A);
    return sweep;
}

/* Eq. 13: P = Q_G [ (Q_G^T grad Q_A) / (v_G v_A^T + gamma) ] Q_A^T, with the
 * eigenvectors in the columns of Q_G, Q_A. */
void oracle_precondition_eigen(const double *QG, const double *vG, const double *QA, const double *vA,
                               const double *grad, int dG, int dA, double gamma, double *P)
{
    double *T1 = (double *)malloc(sizeof(double) * (size_t)dG * dA);
    double *T2 = (double *)malloc(sizeof(double) * (size_t)dG * dA);
    for (int i = 0; i < dG; ++i)            /* T1 = QG^T grad */
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dG; ++k) s += QG[(long)k * dG + i] * grad[(long)k * dA + j];
            T1[(long)i * dA + j] = s;
        }
    for (int i = 0; i < dG; ++i)            /* T2 = (T1 QA) / (vG vA^T + gamma) */
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dA; ++k) s += T1[(long)i * dA + k] * QA[(long)k * dA + j];
            T2[(long)i * dA + j] = s / (vG[i] * vA[j] + gamma);
        }
    for (int i = 0; i < dG; ++i)            /* T1 = QG T2 */
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dG; ++k) s += QG[(long)i * dG + k] * T2[(long)k * dA + j];
            T1[(long)i * dA + j] = s;
        }
    for (int i = 0; i < dG; ++i)            /* P = T1 QA^T */
        for (int j = 0; j < dA; ++j) {
            double s = 0.0;
            for (int k = 0; k < dA; ++k) s += T1[(long)i * dA + k] * QA[(long)j * dA + k];
            P[(long)i * dA + j] = s;
        }
    free(T1); free(T2);
}
