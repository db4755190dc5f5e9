/*
 * lpd_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision CPU statement of what the low-rank stage of
 * the LPD-SVM method (Glasmachers, "Recipe for Fast Large-scale SVM Training",
 * Section 3, Figure 1) computes.  Every function is the definition written
 * out: no blocking, no fusion, no algebraic expansion of the distance, no BLAS.
 * Nothing in the HIP library shares code with this file, and only tests, the
 * smoke check and the CPU-baseline leg of the benchmark may call it.
 *
 * Notation (Figure 1, steps 1a-1d and 2a; Section 4 for the kernel):
 *   landmarks      : B rows of the training set (the "random subset" of 1a)
 *   K_LL  (B x B)  : Gaussian kernel matrix on the landmarks            (1a)
 *   K_LL = U D U^T : symmetric eigendecomposition                       (1b)
 *   U sqrt(D^-1)   : factor of the inverse kernel matrix                (1c)
 *   W (r x B)      : its transpose, W[j,:] = D_j^-1/2 u_j^T -- row j is one
 *                    whitened direction; components whose eigenvalue is below
 *                    tau * D_max are dropped (Section 3, second bullet)
 *   Z (n x B)      : Gaussian kernel between all points and the landmarks (1d)
 *   G = Z W^T      : the low-rank factor, G G^T ~ K                     (1d)
 *   m_i = G_i w    : the margin the coordinate-ascent solver evaluates  (2a)
 *
 * Inputs are the fp32 values the GPU sees, promoted to double on load; all
 * arithmetic and all outputs are double.  OpenMP only spreads independent
 * rows over cores; it changes no summation order inside a row.
 *
 * Pins (tests/test_oracle_pins.py): kernel diagonal = 1, a hand-computed
 * two-point value, scipy's squared-distance routine, G_L G_L^T = K_LL,
 * G_L^T G_L = D, B = n brute force G G^T = K, the projection bound
 * ||g_i||^2 <= 1, the gamma = 0 and duplicated-landmark degenerate cases,
 * LAPACK eigenvalues for the Jacobi solver, unit-vector and landmark-row
 * sweeps for the margins.  The choice of eigenvector basis inside degenerate
 * eigenspaces is a convention (sign and order only): parity unpinned by the
 * paper for that choice, which is why factor parity is taken with one shared W.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Section 4: k(x, x') = exp(-gamma * ||x - x'||^2), by direct differences. */
static double gauss_kernel(const float *x, const float *y, int64_t d, double gamma)
{
    double s = 0.0;
    for (int64_t k = 0; k < d; ++k) {
        double t = (double)x[k] - (double)y[k];
        s += t * t;
    }
    return exp(-gamma * s);
}

/* Figure 1, steps 1a / 1d: the kernel block Z[i,b] = k(x_i, l_b).
 * X: n x d (leading dimension ldx), L: B x d (ldl), Z: n x B dense, double.
 * With X == L and n == B this is K_LL of step 1a. */
void orc_kernel_block(const float *X, int64_t n, int64_t d, int64_t ldx,
                      const float *L, int64_t B, int64_t ldl,
                      double gamma, double *Z)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t b = 0; b < B; ++b)
            Z[i * B + b] = gauss_kernel(X + i * ldx, L + b * ldl, d, gamma);
}

/* Figure 1, step 1b: K = U D U^T by the cyclic two-sided Jacobi method.
 * A (B x B, symmetric, overwritten), V receives eigenvectors as COLUMNS,
 * ev the eigenvalues (unsorted).  Returns the number of sweeps, or -1 if the
 * off-diagonal norm did not fall below 1e-15 * ||A||_F within 60 sweeps. */
int orc_jacobi_eigh(double *A, int64_t B, double *V, double *ev)
{
    double fro = 0.0;
    for (int64_t i = 0; i < B * B; ++i) fro += A[i] * A[i];
    fro = sqrt(fro);
    for (int64_t i = 0; i < B; ++i)
        for (int64_t j = 0; j < B; ++j) V[i * B + j] = (i == j) ? 1.0 : 0.0;

    int sweep;
    for (sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0;
        for (int64_t p = 0; p < B; ++p)
            for (int64_t q = p + 1; q < B; ++q) off += 2.0 * A[p * B + q] * A[p * B + q];
        if (sqrt(off) <= 1e-15 * fro) break;

        for (int64_t p = 0; p < B - 1; ++p) {
            for (int64_t q = p + 1; q < B; ++q) {
                double apq = A[p * B + q];
                if (apq == 0.0) continue;
                /* rotation angle that annihilates A[p,q] */
                double theta = (A[q * B + q] - A[p * B + p]) / (2.0 * apq);
                double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                /* A <- J^T A J with J = rotation in the (p,q) plane */
                for (int64_t k = 0; k < B; ++k) {
                    double akp = A[k * B + p], akq = A[k * B + q];
                    A[k * B + p] = c * akp - s * akq;
                    A[k * B + q] = s * akp + c * akq;
                }
                for (int64_t k = 0; k < B; ++k) {
                    double apk = A[p * B + k], aqk = A[q * B + k];
                    A[p * B + k] = c * apk - s * aqk;
                    A[q * B + k] = s * apk + c * aqk;
                }
                for (int64_t k = 0; k < B; ++k) {
                    double vkp = V[k * B + p], vkq = V[k * B + q];
                    V[k * B + p] = c * vkp - s * vkq;
                    V[k * B + q] = s * vkp + c * vkq;
                }
            }
        }
    }
    for (int64_t i = 0; i < B; ++i) ev[i] = A[i * B + i];
    return sweep < 60 ? sweep : -1;
}

/* Figure 1, step 1c with the dropping rule of Section 3 (second bullet):
 * given eigenpairs (ev[j], column j of V), order them by descending
 * eigenvalue, keep those with ev >= tau * ev_max, fix each kept vector's sign
 * so that its largest-magnitude entry is positive (first such entry on ties),
 * and emit W[j,:] = ev_j^-1/2 * u_j^T.  Rows >= rank of W (B x B) are zero.
 * eig_sorted (may be NULL) receives all B eigenvalues, descending.
 * Returns the rank r (0 if the largest eigenvalue is not positive). */
int64_t orc_whiten_from_eig(const double *V, const double *ev, int64_t B,
                            double tau, double *W, double *eig_sorted)
{
    int64_t *ord = (int64_t *)malloc((size_t)B * sizeof(int64_t));
    for (int64_t i = 0; i < B; ++i) ord[i] = i;
    /* insertion sort, descending, stable */
    for (int64_t i = 1; i < B; ++i) {
        int64_t o = ord[i], j = i;
        while (j > 0 && ev[ord[j - 1]] < ev[o]) { ord[j] = ord[j - 1]; --j; }
        ord[j] = o;
    }
    double evmax = B > 0 ? ev[ord[0]] : 0.0;
    int64_t r = 0;
    memset(W, 0, (size_t)B * (size_t)B * sizeof(double));
    for (int64_t j = 0; j < B; ++j) {
        double lam = ev[ord[j]];
        if (eig_sorted) eig_sorted[j] = lam;
        if (!(evmax > 0.0) || !(lam >= tau * evmax) || !(lam > 0.0)) continue;
        /* kept components are a prefix because the order is descending */
        int64_t col = ord[j];
        double big = 0.0, sgn = 1.0;
        for (int64_t k = 0; k < B; ++k) {
            double v = V[k * B + col];
            if (fabs(v) > big) { big = fabs(v); sgn = v < 0.0 ? -1.0 : 1.0; }
        }
        double scale = sgn / sqrt(lam);
        for (int64_t k = 0; k < B; ++k) W[r * B + k] = scale * V[k * B + col];
        ++r;
    }
    free(ord);
    return r;
}

/* Figure 1, step 1d: G = Z W^T, row by row: g_i = W z_i with
 * z_i[b] = k(x_i, l_b).  W: r x B fp32 (ldw), G: n x r dense double. */
void orc_nystrom_factor(const float *X, int64_t n, int64_t d, int64_t ldx,
                        const float *L, int64_t B, int64_t ldl, double gamma,
                        const float *W, int64_t r, int64_t ldw, double *G)
{
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)(B > 0 ? B : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t b = 0; b < B; ++b)
                z[b] = gauss_kernel(X + i * ldx, L + b * ldl, d, gamma);
            for (int64_t j = 0; j < r; ++j) {
                double s = 0.0;
                for (int64_t b = 0; b < B; ++b) s += (double)W[j * ldw + b] * z[b];
                G[i * r + j] = s;
            }
        }
        free(z);
    }
}

/* Same product with a double-precision W and a precomputed double Z
 * (used by the pins, which work entirely in double). */
void orc_apply_whitening(const double *Z, int64_t n, int64_t B,
                         const double *W, int64_t r, double *G)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < r; ++j) {
            double s = 0.0;
            for (int64_t b = 0; b < B; ++b) s += W[j * B + b] * Z[i * B + b];
            G[i * r + j] = s;
        }
}

/* Figure 1, step 2a: m_i = G_i w = sum_j G[i,j] w[j], j < r.  G is the fp32
 * buffer the solver reads (leading dimension ldg); no label, no offset
 * (the method drops the bias term, Section 2 footnote). */
void orc_margins(const float *G, int64_t n, int64_t r, int64_t ldg,
                 const float *w, double *m)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < r; ++j) s += (double)G[i * ldg + j] * (double)w[j];
        m[i] = s;
    }
}

/* Same sweep over a double G (chained oracle: oracle G -> oracle margins). */
void orc_margins_f64(const double *G, int64_t n, int64_t r, int64_t ldg,
                     const double *w, double *m)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < r; ++j) s += G[i * ldg + j] * w[j];
        m[i] = s;
    }
}

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int t) { omp_set_num_threads(t); }
#else
int orc_num_threads(void) { return 1; }
void orc_set_num_threads(int t) { (void)t; }
#endif
