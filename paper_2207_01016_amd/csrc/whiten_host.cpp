// Host preparation of the low-rank stage (Figure 1 steps 1a-1c, Section 4):
// landmark kernel matrix, symmetric eigendecomposition, inverse-square-root
// factor with small components dropped.  Double precision, OpenMP, no external
// numerical library.
//
// Eigensolver: blocked Householder reduction to tridiagonal form (the symmetric
// matrix-vector products of a panel read the trailing matrix once per column,
// the rank-2*NB update is applied once per panel), implicit-shift QL iteration
// on the tridiagonal matrix with its plane rotations recorded and applied to the
// eigenvector matrix in skewed batches (several QL sweeps share one pass over a
// cache-sized window of vectors), then a blocked back-transformation with the
// Householder reflectors grouped into compact I - V T^T V^T factors.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <vector>

#include "../../include/lpd.h"
#include "whiten_internal.h"

namespace {

constexpr int NB = 32;   // Householder panel width

bool g_verbose = false;  // LPD_VERBOSE=1: progress lines on stderr (long runs are otherwise silent for minutes)

void progress(const char *phase, int64_t done, int64_t total)
{
    static int last_decile = -1;
    if (!g_verbose || total <= 0) return;
    const int decile = int(done * 10 / total);
    if (done == 0) last_decile = -1;
    if (decile != last_decile) {
        last_decile = decile;
        std::fprintf(stderr, "[lpd_whiten_host] %s %d%%\n", phase, decile * 10);
        std::fflush(stderr);
    }
}

inline double sq(double x) { return x * x; }

// ---- step 1a: K[a,b] = exp(-gamma ||l_a - l_b||^2), direct differences, full symmetric storage
void landmark_kernel(const float *L, int64_t B, int64_t d, int64_t ldl, double gamma, double *K)
{
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t a = 0; a < B; ++a) {
        const float *la = L + a * ldl;
        K[a * B + a] = 1.0;
        for (int64_t b = a + 1; b < B; ++b) {
            const float *lb = L + b * ldl;
            double s = 0.0;
#pragma omp simd reduction(+ : s)
            for (int64_t k = 0; k < d; ++k) s += sq(double(la[k]) - double(lb[k]));
            const double v = std::exp(-gamma * s);
            K[a * B + b] = v;
            K[b * B + a] = v;
        }
    }
}

// ---- step 1b, part 1: A = Q T Q^T.
// On exit dg/e hold the tridiagonal matrix (e[j] couples j and j+1), row j of A
// holds the Householder vector v_j in columns j+1.. (v_j[j+1] = 1 implicit value
// stored explicitly), tau[j] its scalar: H_j = I - tau_j v_j v_j^T, Q = H_0 H_1 ...
void tridiagonalise(double *A, int64_t n, double *dg, double *e, double *tau)
{
    std::vector<double> V(size_t(n) * NB), Wm(size_t(n) * NB);   // [row][t]
    std::vector<double> P(size_t(2) * NB * n), Qt(size_t(2) * NB * n);
    std::vector<double> p(n), t1(NB), t2(NB);

    for (int64_t k0 = 0; k0 < n - 2; k0 += NB) {
        progress("tridiagonalisation", k0, n);
        const int nb = int(std::min<int64_t>(NB, n - 2 - k0));
        for (int i = 0; i < nb; ++i) {
            const int64_t j = k0 + i;
            double *row = A + j * n;
            // bring row j (columns j..n-1) up to date with the reflectors of this panel
            if (i > 0) {
#pragma omp parallel for schedule(static) if (n - j > 2048)
                for (int64_t c = j; c < n; ++c) {
                    double s = 0.0;
                    for (int t = 0; t < i; ++t) s += V[j * NB + t] * Wm[c * NB + t] + Wm[j * NB + t] * V[c * NB + t];
                    row[c] -= s;
                }
            }
            dg[j] = row[j];
            // Householder vector from x = row[j+1 .. n-1]
            const int64_t len = n - j - 1;
            double *x = row + j + 1;
            double xnorm2 = 0.0;
            for (int64_t c = 1; c < len; ++c) xnorm2 += sq(x[c]);
            double tj = 0.0, beta = x[0];
            if (xnorm2 > 0.0) {
                const double alpha = x[0];
                beta = -std::copysign(std::sqrt(alpha * alpha + xnorm2), alpha);
                tj = (beta - alpha) / beta;
                const double scal = 1.0 / (alpha - beta);
                for (int64_t c = 1; c < len; ++c) x[c] *= scal;
            }
            x[0] = 1.0;
            e[j] = beta;
            tau[j] = tj;

            // p = tau * (A22 - V W^T - W V^T) v   over rows/cols j+1..n-1
            const double *v = x;   // v[c - (j+1)]
#pragma omp parallel for schedule(static)
            for (int64_t rr = j + 1; rr < n; ++rr) {
                const double *ar = A + rr * n + j + 1;
                double s = 0.0;
#pragma omp simd reduction(+ : s)
                for (int64_t c = 0; c < len; ++c) s += ar[c] * v[c];
                p[rr] = s;
            }
            for (int t = 0; t < i; ++t) t1[t] = t2[t] = 0.0;
            for (int64_t rr = j + 1; rr < n; ++rr) {
                const double vv = v[rr - j - 1];
                for (int t = 0; t < i; ++t) {
                    t1[t] += Wm[rr * NB + t] * vv;
                    t2[t] += V[rr * NB + t] * vv;
                }
            }
            double pv = 0.0;
            for (int64_t rr = j + 1; rr < n; ++rr) {
                double s = p[rr];
                for (int t = 0; t < i; ++t) s -= V[rr * NB + t] * t1[t] + Wm[rr * NB + t] * t2[t];
                s *= tj;
                p[rr] = s;
                pv += s * v[rr - j - 1];
            }
            const double kk = 0.5 * tj * pv;
            for (int64_t rr = 0; rr < n; ++rr) {
                if (rr <= j) {
                    V[rr * NB + i] = 0.0;
                    Wm[rr * NB + i] = 0.0;
                } else {
                    V[rr * NB + i] = v[rr - j - 1];
                    Wm[rr * NB + i] = p[rr] - kk * v[rr - j - 1];
                }
            }
        }
        // trailing update A[s:, s:] -= V W^T + W V^T, s = k0 + nb, as A -= P Qt with
        // P = [V | W] (rows x 2nb) and Qt = [W | V]^T (2nb x cols)
        const int64_t s0 = k0 + nb;
        if (s0 >= n) break;
        const int kk2 = 2 * nb;
        for (int64_t c = s0; c < n; ++c)
            for (int t = 0; t < nb; ++t) {
                Qt[size_t(t) * n + c] = Wm[c * NB + t];
                Qt[size_t(t + nb) * n + c] = V[c * NB + t];
                P[c * kk2 + t] = V[c * NB + t];
                P[c * kk2 + t + nb] = Wm[c * NB + t];
            }
        constexpr int64_t CB = 512;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
        for (int64_t rb = s0; rb < n; rb += 4)
            for (int64_t cb = s0; cb < n; cb += CB) {
                const int64_t ce = std::min(n, cb + CB);
                const int64_t re = std::min(n, rb + 4);
                for (int64_t rr = rb; rr < re; ++rr) {
                    double *ar = A + rr * n;
                    const double *pr = &P[rr * kk2];
                    for (int t = 0; t < kk2; ++t) {
                        const double f = pr[t];
                        const double *q = &Qt[size_t(t) * n];
#pragma omp simd
                        for (int64_t c = cb; c < ce; ++c) ar[c] -= f * q[c];
                    }
                }
            }
    }
    // the last 2x2 block needs no reflector
    if (n >= 2) {
        dg[n - 2] = A[(n - 2) * n + (n - 2)];
        e[n - 2] = A[(n - 2) * n + (n - 1)];
        tau[n - 2] = 0.0;
    }
    if (n >= 1) {
        dg[n - 1] = A[(n - 1) * n + (n - 1)];
        e[n - 1] = 0.0;
        tau[n - 1] = 0.0;
    }
}

// ---- step 1b, part 2: eigen-decomposition of the tridiagonal matrix.
// Zt (n x n) must hold the identity on entry; on exit row i of Zt is the
// eigenvector (in the tridiagonal basis) of eigenvalue dg[i].
using lpd_host::Sweep;

void apply_rotations(double *Zt, int64_t n, const std::vector<Sweep> &sw, const double *cs)
{
    if (sw.empty()) return;
    const int k = int(sw.size());
    int64_t imax = 0, imin = n;
    for (auto &s : sw) { imax = std::max(imax, s.hi); imin = std::min(imin, s.lo); }
    constexpr int64_t SL = 256;   // columns of Zt per task
    const int64_t steps = (imax - imin) + 2 * int64_t(k - 1);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t c0 = 0; c0 < n; c0 += SL) {
        const int64_t c1 = std::min(n, c0 + SL);
        for (int64_t tstep = 0; tstep <= steps; ++tstep) {
            for (int s = 0; s < k; ++s) {
                const int64_t i = imax + 2 * s - tstep;
                if (i > sw[s].hi || i < sw[s].lo) continue;
                const size_t o = sw[s].off + size_t(sw[s].hi - i) * 2;
                const double c = cs[o], sn = cs[o + 1];
                double *zi = Zt + i * n, *zj = Zt + (i + 1) * n;
#pragma omp simd
                for (int64_t q = c0; q < c1; ++q) {
                    const double f = zj[q];
                    zj[q] = sn * zi[q] + c * f;
                    zi[q] = c * zi[q] - sn * f;
                }
            }
        }
    }
}

// ---- step 1b, part 3: rows of Zt become eigenvectors of the original matrix:
// row <- row H_last ... H_1 H_0, reflectors taken NB at a time as I - V T^T V^T.
void back_transform(const double *A, const double *tau, int64_t n, double *Zt)
{
    if (n < 3) return;
    const int64_t nref = n - 2;                 // reflectors 0 .. n-3
    const int64_t npanel = (nref + NB - 1) / NB;
    std::vector<double> T(NB * NB);
    constexpr int64_t RB = 16;                  // rows of Zt per task
    for (int64_t pi = npanel - 1; pi >= 0; --pi) {
        progress("back-transformation", npanel - 1 - pi, npanel);
        const int64_t k0 = pi * NB;
        const int nb = int(std::min<int64_t>(NB, nref - k0));
        const int64_t c0 = k0 + 1;              // first column any reflector of the panel touches
        // v_t lives in A[(k0+t)*n + (k0+t+1) ..]; treat entries left of its start as zero.
        // T upper triangular with H_{k0} ... H_{k0+nb-1} = I - V T V^T.
        std::fill(T.begin(), T.end(), 0.0);
        for (int i = 0; i < nb; ++i) {
            const double ti = tau[k0 + i];
            T[i * NB + i] = ti;
            if (i == 0) continue;
            double z[NB];
            const int64_t si = k0 + i + 1;      // v_i starts here
            for (int t = 0; t < i; ++t) {
                const double *vt = A + (k0 + t) * n;
                const double *vi = A + (k0 + i) * n;
                double s = 0.0;
#pragma omp simd reduction(+ : s)
                for (int64_t c = si; c < n; ++c) s += vt[c] * vi[c];
                z[t] = s;
            }
            for (int a = 0; a < i; ++a) {
                double s = 0.0;
                for (int t = a; t < i; ++t) s += T[a * NB + t] * z[t];
                T[a * NB + i] = -ti * s;
            }
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t r0 = 0; r0 < n; r0 += RB) {
            const int64_t r1 = std::min(n, r0 + RB);
            double Y[RB][NB], Y2[RB][NB];
            for (int64_t rr = r0; rr < r1; ++rr) {
                const double *zr = Zt + rr * n;
                for (int t = 0; t < nb; ++t) {
                    const double *vt = A + (k0 + t) * n;
                    double s = 0.0;
#pragma omp simd reduction(+ : s)
                    for (int64_t c = k0 + t + 1; c < n; ++c) s += zr[c] * vt[c];
                    Y[rr - r0][t] = s;
                }
                // Y2 = Y T^T :  Y2[t] = sum_u Y[u] * T[t][u], T upper => u >= t
                for (int t = 0; t < nb; ++t) {
                    double s = 0.0;
                    for (int u = t; u < nb; ++u) s += Y[rr - r0][u] * T[t * NB + u];
                    Y2[rr - r0][t] = s;
                }
            }
            for (int64_t rr = r0; rr < r1; ++rr) {
                double *zr = Zt + rr * n;
                for (int t = 0; t < nb; ++t) {
                    const double f = Y2[rr - r0][t];
                    const double *vt = A + (k0 + t) * n;
#pragma omp simd
                    for (int64_t c = k0 + t + 1; c < n; ++c) zr[c] -= f * vt[c];
                }
            }
            (void)c0;
        }
    }
}

}  // namespace

namespace lpd_host {

// Implicit-shift QL iteration; returns false if an eigenvalue needs more than 60 sweeps.
bool tridiag_ql(double *dg, double *e, int64_t n, int batch, const RotationBuffer &buffer,
                const ApplyRotations &apply, const std::function<void(int64_t)> &progress)
{
    std::vector<Sweep> sw;
    double *cs = nullptr;       // storage of the current batch, fetched when its first sweep starts
    size_t ncs = 0;
    const double eps = 2.220446049250313e-16;
    for (int64_t l = 0; l < n; ++l) {
        if (progress) progress(l);
        int iter = 0;
        while (true) {
            int64_t m = l;
            for (; m < n - 1; ++m) {
                const double dd = std::fabs(dg[m]) + std::fabs(dg[m + 1]);
                if (std::fabs(e[m]) <= eps * dd) break;
            }
            if (m == l) break;
            if (++iter > 60) return false;
            // Wilkinson-type shift from the leading 2x2 block of the active window
            double g = (dg[l + 1] - dg[l]) / (2.0 * e[l]);
            double r = std::hypot(g, 1.0);
            g = dg[m] - dg[l] + e[l] / (g + std::copysign(r, g));
            double s = 1.0, c = 1.0, p = 0.0;
            if (!cs) {
                cs = buffer();
                if (!cs) return false;
                ncs = 0;
            }
            Sweep rec{m, m - 1, ncs};
            int64_t i = m - 1;
            bool underflow = false;
            for (; i >= l; --i) {
                const double f = s * e[i];
                const double b = c * e[i];
                // sqrt of the plain sum of squares unless it could overflow or lose bits to underflow
                const double rr = f * f + g * g;
                r = (rr > 1e-280 && rr < 1e280) ? std::sqrt(rr) : std::hypot(f, g);
                e[i + 1] = r;
                if (r == 0.0) {
                    dg[i + 1] -= p;
                    e[m] = 0.0;
                    underflow = true;
                    break;
                }
                s = f / r;
                c = g / r;
                g = dg[i + 1] - p;
                r = (dg[i] - g) * s + 2.0 * c * b;
                p = s * r;
                dg[i + 1] = g + p;
                g = c * r - b;
                cs[ncs] = c;
                cs[ncs + 1] = s;
                ncs += 2;
                rec.lo = i;
            }
            if (rec.lo <= rec.hi) sw.push_back(rec);
            if (!underflow) {
                dg[l] -= p;
                e[l] = g;
                e[m] = 0.0;
            }
            if (int(sw.size()) >= batch) {
                apply(sw, cs, ncs);
                sw.clear();
                cs = nullptr;
            }
        }
    }
    if (!sw.empty()) apply(sw, cs, ncs);
    return true;
}

int64_t order_and_clip(const double *dg, int64_t n, double clip_ratio, std::vector<int64_t> &ord, double *eig_sorted)
{
    ord.resize(size_t(n));
    std::iota(ord.begin(), ord.end(), int64_t(0));
    std::stable_sort(ord.begin(), ord.end(), [&](int64_t a, int64_t b) { return dg[a] > dg[b]; });
    if (eig_sorted)
        for (int64_t j = 0; j < n; ++j) eig_sorted[j] = dg[ord[j]];
    if (n == 0) return 0;
    const double top = dg[ord[0]];
    if (!(top > 0.0)) return -1;
    int64_t r = 0;
    while (r < n && dg[ord[r]] >= clip_ratio * top && dg[ord[r]] > 0.0) ++r;
    return r;
}

}  // namespace lpd_host

extern "C" int lpd_whiten_host(const float *L_host, int64_t B, int64_t d, int64_t ldl, double gamma,
                               double clip_ratio, float *W_host, int64_t ldw, double *eig_host, int64_t *rank)
{
    if (B < 0 || d < 0 || B > (int64_t(1) << 20)) return LPD_ERR_SHAPE;
    if (!rank) return LPD_ERR_NULL;
    *rank = 0;
    if (B == 0) return LPD_OK;
    if (!W_host || (d > 0 && !L_host)) return LPD_ERR_NULL;
    if (ldw < B || (d > 0 && ldl < d)) return LPD_ERR_LD;

    const int64_t n = B;
    const char *venv = std::getenv("LPD_VERBOSE");      // progress lines on stderr for long runs
    g_verbose = venv && venv[0] == '1';
    auto say = [&](const char *what) {
        if (g_verbose) { std::fprintf(stderr, "[lpd_whiten_host B=%lld] %s\n", (long long)n, what); std::fflush(stderr); }
    };
    std::vector<double> A(size_t(n) * n), Zt(size_t(n) * n, 0.0), dg(n), e(n), tau(n);
    say("landmark kernel matrix");
    landmark_kernel(L_host, n, d, ldl, gamma, A.data());
    say("tridiagonalisation");
    tridiagonalise(A.data(), n, dg.data(), e.data(), tau.data());
    for (int64_t i = 0; i < n; ++i) Zt[i * n + i] = 1.0;
    say("QL iteration");
    {
        double *zt = Zt.data();
        std::vector<double> store(size_t(32) * 2 * size_t(n));
        auto buffer = [&]() { return store.data(); };
        auto apply = [&](const std::vector<Sweep> &sw, const double *cs, size_t) { apply_rotations(zt, n, sw, cs); };
        auto prog = [&](int64_t l) { progress("QL iteration", l, n); };
        if (!lpd_host::tridiag_ql(dg.data(), e.data(), n, 32, buffer, apply, prog)) return LPD_ERR_NUMERIC;
    }
    say("back-transformation");
    back_transform(A.data(), tau.data(), n, Zt.data());
    say("ordering and scaling");

    std::vector<int64_t> ord;
    const int64_t r = lpd_host::order_and_clip(dg.data(), n, clip_ratio, ord, eig_host);
    if (r < 0) return LPD_ERR_NUMERIC;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        float *wr = W_host + j * ldw;
        if (j >= r) {
            std::memset(wr, 0, size_t(n) * sizeof(float));
            continue;
        }
        const double *u = &Zt[ord[j] * n];
        double big = 0.0, sgn = 1.0;
        for (int64_t k = 0; k < n; ++k)
            if (std::fabs(u[k]) > big) { big = std::fabs(u[k]); sgn = u[k] < 0.0 ? -1.0 : 1.0; }
        const double scale = sgn / std::sqrt(dg[ord[j]]);
        for (int64_t k = 0; k < n; ++k) wr[k] = float(scale * u[k]);
    }
    *rank = r;
    return LPD_OK;
}
