// Driver for the CPU sanitizer tier: runs the host eigensolver of the library (lpd_whiten_host) and every
// function of the CPU oracle on small seeded inputs, including the degenerate shapes, in one executable built
// with -fsanitize=address,undefined.  It checks a few invariants so that the work cannot be optimised away;
// the sanitizers do the real checking.  Built and run by tests/test_sanitizers_cpu.py.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int lpd_whiten_host(const float *L_host, int64_t B, int64_t d, int64_t ldl, double gamma, double clip_ratio,
                    float *W_host, int64_t ldw, double *eig_host, int64_t *rank);
void orc_kernel_block(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                      double gamma, double *Z);
void orc_kernel_block_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values, int64_t n, int64_t d,
                          const float *L, int64_t B, int64_t ldl, double gamma, double *Z);
int orc_jacobi_eigh(double *A, int64_t B, double *V, double *ev);
int64_t orc_whiten_from_eig(const double *V, const double *ev, int64_t B, double tau, double *W, double *eig_sorted);
void orc_nystrom_factor(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                        double gamma, const float *W, int64_t r, int64_t ldw, double *G);
void orc_apply_whitening(const double *Z, int64_t n, int64_t B, const double *W, int64_t r, double *G);
void orc_margins(const float *G, int64_t n, int64_t r, int64_t ldg, const float *w, double *m);
void orc_margins_f64(const double *G, int64_t n, int64_t r, int64_t ldg, const double *w, double *m);
void orc_cd_solve(const float *G, int64_t r, int64_t ldg, const int64_t *rows, const float *y, int64_t np, double C,
                  double eps, int64_t max_epochs, int64_t shrink_k, double eta, double *alpha, double *w,
                  double *stats);
void orc_predict(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                 double gamma, const float *W, int64_t r, int64_t ldw, const float *Ws, int64_t c, int64_t ldws,
                 double *F);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static float rnd()
{
    g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
    return float(double(g_state >> 11) / double(1ull << 53)) * 2.0f - 1.0f;
}

static int fail(const char *what) { std::fprintf(stderr, "sanitize_driver: %s\n", what); return 1; }

static int host_whiten_case(int64_t B, int64_t d, double gamma, bool duplicate)
{
    const int64_t ldl = d + 3, ldw = B + 1;
    std::vector<float> L((size_t)(B > 0 ? B : 1) * ldl), W((size_t)(B > 0 ? B : 1) * ldw);
    for (auto &v : L) v = rnd();
    if (duplicate && B > 1)
        for (int64_t k = 0; k < d; ++k) L[(size_t)(B - 1) * ldl + k] = L[k];
    std::vector<double> eig((size_t)(B > 0 ? B : 1));
    int64_t rank = -1;
    const int st = lpd_whiten_host(L.data(), B, d, ldl, gamma, 1e-10, W.data(), ldw, eig.data(), &rank);
    if (st != 0) return fail("lpd_whiten_host status");
    if (rank < 0 || rank > B) return fail("lpd_whiten_host rank");
    double tr = 0.0;
    for (int64_t j = 0; j < B; ++j) tr += eig[(size_t)(j)];
    if (B > 0 && std::fabs(tr - double(B)) > 1e-8 * double(B)) return fail("trace of the kernel matrix");
    if (duplicate && B > 1 && rank != B - 1) return fail("duplicate landmark not dropped");
    if (gamma == 0.0 && B > 0 && rank != 1) return fail("gamma = 0 must have rank 1");
    return 0;
}

int main(int argc, char **argv)
{
    if (argc > 1 && argv[1][0] == 'p') {
        // planted mistake, to show that the sanitizers of this build are live: the kernel block of 3 x 3
        // points written into room for 8 values
        std::vector<float> P(6, 0.5f);
        double *small = static_cast<double *>(std::malloc(8 * sizeof(double)));
        orc_kernel_block(P.data(), 3, 2, 2, P.data(), 3, 2, 0.1, small);
        std::free(small);
        return 0;
    }
    // ---- host eigensolver of the library: sizes around its panel width (32) and batch sizes, degenerate cases
    for (int64_t B : {0, 1, 2, 3, 31, 32, 33, 64, 97, 200, 333})
        if (host_whiten_case(B, 5, 0.3, false)) return 1;
    if (host_whiten_case(40, 4, 0.0, false)) return 1;
    if (host_whiten_case(65, 6, 0.2, true)) return 1;
    if (host_whiten_case(7, 0, 0.5, false) == 0) { /* d = 0: all points coincide, rank 1 expected or refused */ }

    // ---- oracle: kernel block, eigensolver, whitening, factor, margins
    const int64_t n = 57, d = 7, B = 19;
    std::vector<float> X((size_t)(n) * d), L((size_t)(B) * d);
    for (auto &v : X) v = rnd();
    for (int64_t b = 0; b < B; ++b)
        for (int64_t k = 0; k < d; ++k) L[(size_t)(b) * d + k] = X[(size_t)(b * 3) * d + k];
    std::vector<double> K((size_t)(B) * B), Kc, V((size_t)(B) * B), ev((size_t)(B)), Wd((size_t)(B) * B), es((size_t)(B));
    orc_kernel_block(L.data(), B, d, d, L.data(), B, d, 0.4, K.data());
    for (int64_t b = 0; b < B; ++b)
        if (K[(size_t)(b) * B + b] != 1.0) return fail("kernel diagonal");
    Kc = K;
    if (orc_jacobi_eigh(Kc.data(), B, V.data(), ev.data()) < 0) return fail("jacobi");
    const int64_t r = orc_whiten_from_eig(V.data(), ev.data(), B, 1e-10, Wd.data(), es.data());
    if (r != B) return fail("oracle rank");
    std::vector<float> W32((size_t)(B) * B);
    for (size_t i = 0; i < W32.size(); ++i) W32[i] = float(Wd[i]);
    std::vector<double> G((size_t)(n) * r), Z((size_t)(n) * B), G2((size_t)(n) * r), m((size_t)(n)), m2((size_t)(n));
    orc_nystrom_factor(X.data(), n, d, d, L.data(), B, d, 0.4, W32.data(), r, B, G.data());
    orc_kernel_block(X.data(), n, d, d, L.data(), B, d, 0.4, Z.data());
    orc_apply_whitening(Z.data(), n, B, Wd.data(), r, G2.data());
    for (size_t i = 0; i < G.size(); ++i)
        if (std::fabs(G[i] - G2[i]) > 1e-5) return fail("factor by two routes");
    std::vector<float> G32(G.size()), w((size_t)(r));
    std::vector<double> wd((size_t)(r));
    for (size_t i = 0; i < G.size(); ++i) G32[i] = float(G[i]);
    for (int64_t j = 0; j < r; ++j) { w[(size_t)(j)] = rnd(); wd[(size_t)(j)] = w[(size_t)(j)]; }
    orc_margins(G32.data(), n, r, r, w.data(), m.data());
    orc_margins_f64(G.data(), n, r, r, wd.data(), m2.data());
    for (int64_t i = 0; i < n; ++i)
        if (std::fabs(m[(size_t)(i)] - m2[(size_t)(i)]) > 1e-5) return fail("margins");

    // ---- oracle: compressed rows (empty rows, unsorted columns)
    {
        std::vector<int64_t> rp{0};
        std::vector<int32_t> ci;
        std::vector<float> va;
        std::vector<float> Xd((size_t)(n) * d, 0.0f);
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t k = d - 1; k >= 0; --k)
                if (i % 5 != 0 && rnd() > 0.2f) { ci.push_back(int32_t(k)); va.push_back(rnd()); Xd[(size_t)(i) * d + k] = va.back(); }
            rp.push_back(int64_t(ci.size()));
        }
        std::vector<double> Zs((size_t)(n) * B), Zd((size_t)(n) * B);
        orc_kernel_block_csr(rp.data(), ci.data(), va.data(), n, d, L.data(), B, d, 0.4, Zs.data());
        orc_kernel_block(Xd.data(), n, d, d, L.data(), B, d, 0.4, Zd.data());
        for (size_t i = 0; i < Zs.size(); ++i)
            if (Zs[i] != Zd[i]) return fail("compressed rows against dense");
    }

    // ---- oracle: solver (shrinking on and off, warm start, a zero row, one variable, none) and prediction
    {
        std::vector<int64_t> rows((size_t)(n));
        std::vector<float> y((size_t)(n));
        for (int64_t i = 0; i < n; ++i) { rows[(size_t)(i)] = (i * 7) % n; y[(size_t)(i)] = rnd() > 0 ? 1.0f : -1.0f; }
        for (int64_t j = 0; j < r; ++j) G32[(size_t)(5) * r + j] = 0.0f;
        std::vector<double> alpha((size_t)(n), 0.0), ww((size_t)(r)), stats(6);
        for (int64_t k : {int64_t(0), int64_t(2), int64_t(5)}) {
            orc_cd_solve(G32.data(), r, r, rows.data(), y.data(), n, 1.0, 1e-6, 100000, k, 0.05, alpha.data(), ww.data(),
                         stats.data());
            if (stats[2] != 1.0) return fail("solver did not converge");
        }
        orc_cd_solve(G32.data(), r, r, rows.data(), y.data(), n, 1.0, 1e-6, 100000, 5, 0.5, alpha.data(), ww.data(),
                     stats.data());                                   // warm start, a re-check after every step
        orc_cd_solve(G32.data(), r, r, rows.data(), y.data(), 1, 1.0, 1e-6, 10, 5, 0.05, alpha.data(), ww.data(), stats.data());
        orc_cd_solve(G32.data(), r, r, rows.data(), y.data(), 0, 1.0, 1e-6, 10, 5, 0.05, alpha.data(), ww.data(), stats.data());
        std::vector<float> Ws((size_t)(3) * r);
        for (auto &v : Ws) v = rnd();
        std::vector<double> F((size_t)(n) * 3);
        orc_predict(X.data(), n, d, d, L.data(), B, d, 0.4, W32.data(), r, B, Ws.data(), 3, r, F.data());
        if (!std::isfinite(F[0])) return fail("prediction");
    }
    std::puts("sanitize_driver: ok");
    return 0;
}
