/*
 * lpd_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision CPU statement of what the low-rank stage of
 * the LPD-SVM method (Glasmachers, "Recipe for Fast Large-scale SVM Training",
 * Section 4, Figure 1) computes.  Every function is the definition written
 * out: no blocking, no fusion, no algebraic expansion of the distance, no BLAS.
 * Nothing in the HIP library shares code with this file, and only tests, the
 * smoke check and the CPU-baseline leg of the benchmark may call it.
 *
 * Notation (Figure 1, steps 1a-1d and 2a; Section 5 for the kernel):
 *   landmarks      : B rows of the training set (the "random subset" of 1a)
 *   K_LL  (B x B)  : Gaussian kernel matrix on the landmarks            (1a)
 *   K_LL = U D U^T : symmetric eigendecomposition                       (1b)
 *   U sqrt(D^-1)   : factor of the inverse kernel matrix                (1c)
 *   W (r x B)      : its transpose, W[j,:] = D_j^-1/2 u_j^T -- row j is one
 *                    whitened direction; components whose eigenvalue is below
 *                    tau * D_max are dropped (Section 4, second bullet)
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

/* Section 5: k(x, x') = exp(-gamma * ||x - x'||^2), by direct differences. */
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

/* The kernel block for sparse inputs (Section 4, "Multi-core and GPU
 * Implementation": every kernel operation of the method also runs on sparse
 * data, through sparse matrix products): row i of X is given
 * in compressed-row form, entries row_ptr[i] .. row_ptr[i+1]-1 of (col_idx,
 * values), every other coordinate zero; column indices of a row are distinct,
 * in any order.  The kernel value is that of the vector so described:
 * the row is written out in full and the definition applied. */
void orc_kernel_block_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values,
                          int64_t n, int64_t d,
                          const float *L, int64_t B, int64_t ldl,
                          double gamma, double *Z)
{
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(d > 0 ? d : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t k = 0; k < d; ++k) x[k] = 0.0;
            for (int64_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) x[col_idx[e]] = (double)values[e];
            for (int64_t b = 0; b < B; ++b) {
                const float *l = L + b * ldl;
                double s = 0.0;
                for (int64_t k = 0; k < d; ++k) {
                    const double df = x[k] - (double)l[k];
                    s += df * df;
                }
                Z[i * B + b] = exp(-gamma * s);
            }
        }
        free(x);
    }
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

/* Figure 1, step 1c with the dropping rule of Section 4 (second bullet):
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

/* ------------------------------------------------------------------------
 * Stage 2: dual coordinate ascent on the linear problem whose data points are
 * the rows of G (Section 2, equation (2) and the truncated Newton step;
 * Section 4, "Shrinking"; Figure 1 steps 2a-2b).
 *
 *   maximise  D(alpha) = sum_i alpha_i - 1/2 ||w||^2,   0 <= alpha_i <= C,
 *   w = sum_i alpha_i y_i g_i,   Q_ij = y_i y_j g_i . g_j
 *
 * One step on variable i (2a, 2b):
 *   f = g_i . w ;  grad = 1 - y_i f ;  alpha_i <- clip(alpha_i + grad / Q_ii, 0, C) ;
 *   w <- w + (alpha_new - alpha_old) y_i g_i.
 * A row with Q_ii = 0 cannot change w; its alpha goes to C (grad = 1 > 0).
 *
 * Section 4, "Shrinking", fixes k = 5 and eta = 5 % and says no more about how
 * the eta share is spent; the stopping criterion is named (Section 4, third
 * point of the comparison with LLSVM) as a standard one of the kind the
 * linear-SVM dual solvers use, and not spelled out.  Where the text is silent
 * this file takes the plainest sequential reading:
 *   - variables are visited round-robin in the order of the active list, which
 *     starts as the caller's order; an epoch is one pass over that list;
 *   - a variable whose step left alpha exactly unchanged k times in a row is
 *     removed (appended to a FIFO queue of removed variables);
 *   - after every S = round((1 - eta) / eta) steps on active variables one step
 *     is spent on the head of that queue: if the step changes alpha the variable
 *     is reactivated (joins the next epoch's list), otherwise it returns to the
 *     tail.  Every step costs one inner product, so a fraction eta of the work
 *     goes into re-checking removed variables;
 *   - KKT violation of a variable, measured before its step: max(grad, 0) at
 *     alpha = 0, max(-grad, 0) at alpha = C, |grad| inside;
 *   - stopping, in two parts as in the dual linear solvers the paper points to
 *     (criterion met on the shrunk problem, then confirmed on the whole one):
 *     when the largest violation seen in an epoch is <= eps, w is set to its
 *     definition sum_i alpha_i y_i g_i and all removed variables are checked
 *     with that w (a margin sweep over their rows, step 2a); those violating by
 *     more than eps are reactivated.  The solver stops when there are none AND
 *     the epoch that met the criterion had itself started from such a w, i.e.
 *     the criterion is confirmed by one whole epoch in which every active
 *     variable was measured against w = sum alpha y g and not against the sum
 *     of all increments since the start.  The first epoch qualifies (the start
 *     w is computed from the start alpha).  In exact arithmetic the confirming
 *     epoch changes nothing but costs its steps; they are counted.
 *
 * G: fp32 factor (ldg), rows/y: the problem's np variables in visiting order,
 * alpha: in (warm start) / out, w: out (r doubles).  stats (6 doubles): epochs,
 * steps (inner products spent), converged (0/1), final active count, last
 * epoch's largest violation, dual objective.
 * ------------------------------------------------------------------------ */
static double orc_dot_row(const float *g, const double *w, int64_t r)
{
    double s = 0.0;
    for (int64_t j = 0; j < r; ++j) s += (double)g[j] * w[j];
    return s;
}

static double orc_violation(double alpha, double grad, double C)
{
    if (alpha <= 0.0) return grad > 0.0 ? grad : 0.0;
    if (alpha >= C) return grad < 0.0 ? -grad : 0.0;
    return fabs(grad);
}

void orc_cd_solve(const float *G, int64_t r, int64_t ldg,
                  const int64_t *rows, const float *y, int64_t np, double C,
                  double eps, int64_t max_epochs, int64_t shrink_k, double eta,
                  double *alpha, double *w, double *stats)
{
    int64_t *act = (int64_t *)malloc((size_t)(np + 1) * sizeof(int64_t));
    int64_t *nxt = (int64_t *)malloc((size_t)(np + 1) * sizeof(int64_t));
    int64_t *rem = (int64_t *)malloc((size_t)(np + 1) * sizeof(int64_t));   /* circular FIFO */
    int64_t *cnt = (int64_t *)calloc((size_t)(np + 1), sizeof(int64_t));
    int64_t n_act = np, n_rem = 0, head = 0, steps = 0, since = 0, epochs = 0;
    int converged = 0, fresh = 1;   /* the start w is computed from the start alpha */
    double maxviol = 0.0;
    const int64_t S = eta > 0.0 ? (int64_t)floor((1.0 - eta) / eta + 0.5) : 0;

    for (int64_t j = 0; j < r; ++j) w[j] = 0.0;
    for (int64_t t = 0; t < np; ++t) {
        act[t] = t;
        if (alpha[t] != 0.0) {
            const float *g = G + rows[t] * ldg;
            for (int64_t j = 0; j < r; ++j) w[j] += alpha[t] * (double)y[t] * (double)g[j];
        }
    }

    while (epochs < max_epochs && !converged) {
        int64_t n_nxt = 0;
        maxviol = 0.0;
        for (int64_t pos = 0; pos < n_act; ++pos) {
            /* the eta share: one step on the head of the removed queue */
            if (shrink_k > 0 && S > 0 && since >= S && n_rem > 0) {
                const int64_t t = rem[head];
                head = (head + 1) % (np + 1);
                --n_rem;
                const float *g = G + rows[t] * ldg;
                double q = 0.0;
                for (int64_t j = 0; j < r; ++j) q += (double)g[j] * (double)g[j];
                const double grad = 1.0 - (double)y[t] * orc_dot_row(g, w, r);
                double an = q > 0.0 ? alpha[t] + grad / q : C;
                an = an < 0.0 ? 0.0 : (an > C ? C : an);
                ++steps;
                since = 0;
                if (an != alpha[t]) {
                    const double dl = (an - alpha[t]) * (double)y[t];
                    for (int64_t j = 0; j < r; ++j) w[j] += dl * (double)g[j];
                    alpha[t] = an;
                    cnt[t] = 0;
                    nxt[n_nxt++] = t;
                } else {
                    rem[(head + n_rem) % (np + 1)] = t;
                    ++n_rem;
                }
            }
            const int64_t t = act[pos];
            const float *g = G + rows[t] * ldg;
            double q = 0.0;
            for (int64_t j = 0; j < r; ++j) q += (double)g[j] * (double)g[j];
            const double grad = 1.0 - (double)y[t] * orc_dot_row(g, w, r);   /* step 2a */
            const double v = orc_violation(alpha[t], grad, C);
            if (v > maxviol) maxviol = v;
            double an = q > 0.0 ? alpha[t] + grad / q : C;                   /* step 2b */
            an = an < 0.0 ? 0.0 : (an > C ? C : an);
            ++steps;
            ++since;
            if (an != alpha[t]) {
                const double dl = (an - alpha[t]) * (double)y[t];
                for (int64_t j = 0; j < r; ++j) w[j] += dl * (double)g[j];
                alpha[t] = an;
                cnt[t] = 0;
                nxt[n_nxt++] = t;
            } else if (shrink_k > 0 && ++cnt[t] >= shrink_k) {
                rem[(head + n_rem) % (np + 1)] = t;
                ++n_rem;
            } else {
                nxt[n_nxt++] = t;
            }
        }
        ++epochs;
        if (maxviol <= eps) {
            /* recompute w from alpha (sheds the rounding drift of the incremental updates; a
             * no-op in exact arithmetic), then sweep over the removed variables with w fixed */
            for (int64_t j = 0; j < r; ++j) w[j] = 0.0;
            for (int64_t t = 0; t < np; ++t) {
                if (alpha[t] == 0.0) continue;
                const float *g = G + rows[t] * ldg;
                for (int64_t j = 0; j < r; ++j) w[j] += alpha[t] * (double)y[t] * (double)g[j];
                ++steps;
            }
            int64_t back = 0;
            const int64_t m = n_rem;
            for (int64_t c = 0; c < m; ++c) {
                const int64_t t = rem[head];
                head = (head + 1) % (np + 1);
                --n_rem;
                const float *g = G + rows[t] * ldg;
                const double grad = 1.0 - (double)y[t] * orc_dot_row(g, w, r);
                ++steps;
                if (orc_violation(alpha[t], grad, C) > eps) {
                    cnt[t] = 0;
                    nxt[n_nxt++] = t;
                    ++back;
                } else {
                    rem[(head + n_rem) % (np + 1)] = t;
                    ++n_rem;
                }
            }
            if (back == 0 && fresh) converged = 1;   /* the epoch itself started from a recomputed w */
            fresh = 1;
        } else {
            fresh = 0;
        }
        { int64_t *tmp = act; act = nxt; nxt = tmp; }
        n_act = n_nxt;
    }
    double sa = 0.0, ww = 0.0;
    for (int64_t t = 0; t < np; ++t) sa += alpha[t];
    for (int64_t j = 0; j < r; ++j) ww += w[j] * w[j];
    stats[0] = (double)epochs;
    stats[1] = (double)steps;
    stats[2] = (double)converged;
    stats[3] = (double)n_act;
    stats[4] = maxviol;
    stats[5] = sa - 0.5 * ww;
    free(act); free(nxt); free(rem); free(cnt);
}

/* ------------------------------------------------------------------------
 * Prediction (Section 4, "Algorithm Overview": the prediction step; Section 2:
 * f(x) = <w, phi(x)>, no offset).  In the low-rank feature space the features of
 * a new point x are g(x) = W z(x), z(x)_b = k(x, l_b) -- the same map that
 * produced the rows of G (Figure 1, 1d) -- and classifier j scores it with
 * f_j(x) = ws_j . g(x) (Figure 1, 2a).  Written out exactly so: kernel row by
 * direct differences, then W, then the weight vectors; nothing is folded.
 * X: n x d, L: B x d, W: r x B (ldw), Ws: c x r (ldws), F: n x c double.
 * ------------------------------------------------------------------------ */
void orc_predict(const float *X, int64_t n, int64_t d, int64_t ldx,
                 const float *L, int64_t B, int64_t ldl, double gamma,
                 const float *W, int64_t r, int64_t ldw,
                 const float *Ws, int64_t c, int64_t ldws, double *F)
{
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)(B > 0 ? B : 1) * sizeof(double));
        double *g = (double *)malloc((size_t)(r > 0 ? r : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t b = 0; b < B; ++b)
                z[b] = gauss_kernel(X + i * ldx, L + b * ldl, d, gamma);
            for (int64_t j = 0; j < r; ++j) {
                double s = 0.0;
                for (int64_t b = 0; b < B; ++b) s += (double)W[j * ldw + b] * z[b];
                g[j] = s;
            }
            for (int64_t q = 0; q < c; ++q) {
                double s = 0.0;
                for (int64_t j = 0; j < r; ++j) s += (double)Ws[q * ldws + j] * g[j];
                F[i * c + q] = s;
            }
        }
        free(z);
        free(g);
    }
}
