// Stage-1 preparation on the device (Figure 1 steps 1a-1c, Section 4): landmark kernel matrix,
// symmetric eigendecomposition and the whitening factor W = Lambda^{-1/2} U^T, in double precision,
// for gfx950.  All O(B^3) work runs in the kernels below; the host keeps only the serial scalar part,
// the implicit-shift QL iteration on the tridiagonal matrix (O(B^2)), and overlaps it with the device.
//
//   1a  kll_kernel        K[a,b] = exp(-gamma ||l_a - l_b||^2) from direct differences
//   1b  rowfix / hh / symv / pfix / w kernels per column, syr2k_kernel per panel of 32 columns: blocked
//       Householder reduction to tridiagonal form.  A column reads the trailing matrix once (8 bytes
//       per element, the pass that bounds the reduction); the matrix is rewritten once per panel.
//       panel_gram_kernel / panel_t_kernel / panel_apply_kernel: Q^T accumulated row-wise from the
//       reflectors, 32 at a time in compact form I - V T^T V^T.
//       rot_table_kernel / rot_kernel: the QL plane rotations, 16 sweeps per pass.  A lane owns one
//       column of the eigenvector matrix; the sweeps form a pipeline of 16 stages (registers inside a
//       wavefront, LDS between the four wavefronts of a workgroup): rows enter in descending order,
//       a stage holds one row, rotates it against the next and hands it on two steps later, so the
//       rotations of a step are independent and a pass reads and writes each row once.
//   1c  finish_kernel     W[j,:] = sign_j * u_j / sqrt(lambda_j) in eigenvalue order, rows >= r zero.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <numeric>
#include <thread>
#include <vector>

#include "../../include/lpd.h"
#include "whiten_internal.h"

namespace {

constexpr int NB = 32;        // reflectors per compact panel
constexpr int KSW = 16;       // QL sweeps per rotation pass
constexpr size_t kAlign = 256;

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum over a workgroup of up to 1024 threads; every thread gets the result. `red` holds 16 doubles.
__device__ __forceinline__ double block_sum(double v, double *red)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int k = 0; k < nw; ++k) t += red[k];
    return t;
}

// ---------------------------------------------------------------- step 1a

__global__ __launch_bounds__(256) void kll_kernel(const float *__restrict__ L, int n, int d, int64_t ldl, double gamma,
                                                  double *__restrict__ A)
{
    __shared__ float la[16][33], lb[16][33];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int a0 = blockIdx.y * 16, b0 = blockIdx.x * 16;
    double s = 0.0;
    for (int k0 = 0; k0 < d; k0 += 32) {
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * 32; e += 256) {
            const int r = e >> 5, k = e & 31;
            la[r][k] = (a0 + r < n && k0 + k < d) ? L[int64_t(a0 + r) * ldl + k0 + k] : 0.f;
            lb[r][k] = (b0 + r < n && k0 + k < d) ? L[int64_t(b0 + r) * ldl + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            const double df = double(la[ty][k]) - double(lb[tx][k]);
            s += df * df;
        }
    }
    const int a = a0 + ty, b = b0 + tx;
    if (a < n && b < n) A[int64_t(a) * n + b] = a == b ? 1.0 : exp(-gamma * s);
}

// ---------------------------------------------------------------- step 1b, tridiagonalisation
//
// Blocked Householder reduction.  Inside a panel of NBT columns the trailing matrix is left as it was
// when the panel began (A_old); what the panel's reflectors have done to it so far lives in the pairs
// (v_k, w_k) of the panel, A_cur = A_old - sum_k (v_k w_k^T + w_k v_k^T).  A column therefore costs one
// READ of the trailing matrix (symv_kernel, 8 bytes per element) plus thin corrections with the panel's
// vectors; the trailing matrix is rewritten once per panel (syr2k_kernel).
// Per column j = j0 + i:   rowfix (current row j)  ->  hh (reflector v_i, tau, e_j, d_j)
//                          ->  symv (y = A_old v_i; a_k = w_k . v_i, b_k = v_k . v_i for k < i)
//                          ->  pfix (y -= sum_k v_k a_k + w_k b_k)  ->  w (w_i from y)

constexpr int NBT = 32;       // columns per panel of the reduction

typedef double d2 __attribute__((ext_vector_type(2)));

// x[c] = A_old[j, c] - sum_{k<i} (v_k[j] w_k[c] + w_k[j] v_k[c]) for c >= j: row j as it stands now.
__global__ __launch_bounds__(256) void rowfix_kernel(const double *__restrict__ A, int n, int j, int i,
                                                     const double *__restrict__ Vp, const double *__restrict__ Wp,
                                                     double *__restrict__ x)
{
    const int c = j + blockIdx.x * 256 + threadIdx.x;
    if (c >= n) return;
    double v = A[int64_t(j) * n + c];
    for (int k = 0; k < i; ++k) {
        const double *vk = Vp + int64_t(k) * n, *wk = Wp + int64_t(k) * n;
        v -= vk[j] * wk[c] + wk[j] * vk[c];
    }
    x[c] = v;
}

// One workgroup.  From the current row x (columns j..): d_j = x[j], the Householder vector v over columns
// j+1.. (v[j+1] = 1) with H x[j+1..] = e_j * unit vector, tau_j.  v goes to vout (the panel) and over row j
// of A, where the accumulation of Q finds it later.
__global__ __launch_bounds__(1024) void hh_kernel(double *__restrict__ A, int n, int j, const double *__restrict__ x,
                                                  double *__restrict__ vout, double *__restrict__ dg,
                                                  double *__restrict__ e, double *__restrict__ tau)
{
    __shared__ double red[16];
    double *row = A + int64_t(j) * n;
    double ss = 0.0;
    for (int c = j + 2 + threadIdx.x; c < n; c += blockDim.x) ss += x[c] * x[c];
    ss = block_sum(ss, red);
    const double diag = x[j], alpha = x[j + 1];
    double beta = alpha, t = 0.0, scale = 0.0;
    if (ss > 0.0) {
        beta = -copysign(sqrt(alpha * alpha + ss), alpha);
        t = (beta - alpha) / beta;
        scale = 1.0 / (alpha - beta);
    }
    for (int c = j + 1 + threadIdx.x; c < n; c += blockDim.x) {
        const double v = c == j + 1 ? 1.0 : x[c] * scale;
        vout[c] = v;
        row[c] = v;
    }
    if (threadIdx.x == 0) {
        dg[j] = diag;
        e[j] = beta;
        tau[j] = t;
    }
}

// y[a] = sum_{c > j} A_old[a, c] v[c] for rows a > j: read-only pass over the trailing matrix, one
// wavefront per row pair (VEC: n even, 16-byte accesses from the even column at or below j+1, the element
// left of j+1 masked) or per row.  Workgroups past the rows (blockIdx.x >= row_blocks) compute the panel
// dots instead: block row_blocks + k gives coef[2k] = w_k . v and coef[2k+1] = v_k . v.
template <bool VEC>
__global__ __launch_bounds__(256) void symv_kernel(const double *__restrict__ A, int n, int j, int row_blocks,
                                                   const double *__restrict__ v, double *__restrict__ y,
                                                   const double *__restrict__ Vp, const double *__restrict__ Wp,
                                                   double *__restrict__ coef)
{
    const int lane = threadIdx.x & 63;
    const int c0 = j + 1;
    if (int(blockIdx.x) >= row_blocks) {
        __shared__ double red[16];
        const int k = blockIdx.x - row_blocks;
        const double *vk = Vp + int64_t(k) * n, *wk = Wp + int64_t(k) * n;
        double sa = 0.0, sb = 0.0;
        for (int c = c0 + threadIdx.x; c < n; c += 256) {
            const double vc = v[c];
            sa += wk[c] * vc;
            sb += vk[c] * vc;
        }
        sa = block_sum(sa, red);
        sb = block_sum(sb, red);
        if (threadIdx.x == 0) { coef[2 * k] = sa; coef[2 * k + 1] = sb; }
        return;
    }
    if (VEC) {
        const int cal = c0 & ~1;
        const int npair = (n - c0 + 1) / 2;
        for (int pr = blockIdx.x * 4 + (threadIdx.x >> 6); pr < npair; pr += row_blocks * 4) {
            const int a0 = c0 + 2 * pr;
            const bool two = a0 + 1 < n;
            const double *r0 = A + int64_t(a0) * n, *r1 = A + int64_t(two ? a0 + 1 : a0) * n;
            double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
            int c = cal + 2 * lane;
            if (c < n) {        // first slice: the element left of j+1 carries no weight
                d2 vv = *reinterpret_cast<const d2 *>(v + c);
                if (c < c0) vv.x = 0.0;
                const d2 x0 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r0 + c));
                const d2 x1 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r1 + c));
                acc0 += x0.x * vv.x + x0.y * vv.y;
                acc1 += x1.x * vv.x + x1.y * vv.y;
                c += 128;
            }
            for (; c + 128 < n; c += 256) {
                const d2 va = *reinterpret_cast<const d2 *>(v + c), vb = *reinterpret_cast<const d2 *>(v + c + 128);
                const d2 x0 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r0 + c));
                const d2 x1 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r1 + c));
                const d2 x2 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r0 + c + 128));
                const d2 x3 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r1 + c + 128));
                acc0 += x0.x * va.x + x0.y * va.y;
                acc1 += x1.x * va.x + x1.y * va.y;
                acc2 += x2.x * vb.x + x2.y * vb.y;
                acc3 += x3.x * vb.x + x3.y * vb.y;
            }
            if (c < n) {
                const d2 va = *reinterpret_cast<const d2 *>(v + c);
                const d2 x0 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r0 + c));
                const d2 x1 = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(r1 + c));
                acc0 += x0.x * va.x + x0.y * va.y;
                acc1 += x1.x * va.x + x1.y * va.y;
            }
            acc0 = wave_sum(acc0 + acc2);
            acc1 = wave_sum(acc1 + acc3);
            if (lane == 0) {
                y[a0] = acc0;
                if (two) y[a0 + 1] = acc1;
            }
        }
    } else {
        for (int a = c0 + blockIdx.x * 4 + (threadIdx.x >> 6); a < n; a += row_blocks * 4) {
            const double *row = A + int64_t(a) * n;
            double acc = 0.0;
            for (int c = c0 + lane; c < n; c += 64) acc += row[c] * v[c];
            acc = wave_sum(acc);
            if (lane == 0) y[a] = acc;
        }
    }
}

// The same product from the UPPER triangle alone: the trailing matrix is symmetric, so an element A[a, c],
// c > a, serves row a (times v[c]) and row c (times v[a]) in one read, and the pass reads half the bytes.
// Work item = a strip of 64 rows (16 per wavefront) times a segment of `nch` chunks of 128 columns (4 chunks;
// 2 once the trailing matrix has 8,192 rows or fewer, so that the strips left still make enough workgroups and
// each one's serial walk, a memory round trip per chunk, is short; 8 chunks measured 2 % slower at 16,384 rows); a lane holds 2 columns of the chunk and 16 row sums.  Row sums of a segment go to
// rowpart[segment][row]; the column sums of a chunk are combined over the four wavefronts in LDS and go to
// colpart[strip][column]; yfix_kernel adds both up in a fixed order (no atomics: the result does not depend
// on the order in which workgroups finish).  Elements left of the diagonal are read with their chunk and
// masked; they are never meant: the panel update (syr2k_kernel) maintains the upper triangle only.
// blockIdx.y >= n_strips: the panel dots, as in symv_kernel.
constexpr int SY_ROWS = 64, SY_WR = 16, SY_CH = 128, SY_NCH = 4, SY_SEG = SY_CH * SY_NCH;
constexpr int SY_SMALL = 8192, SY_NCH_SMALL = 2;     // trailing matrices of up to SY_SMALL rows: segments of 2 chunks

template <bool VEC>
__global__ __launch_bounds__(256) void symv_upper_kernel(const double *__restrict__ A, int n, int j, int n_strips,
                                                         const double *__restrict__ v, double *__restrict__ rowpart,
                                                         double *__restrict__ colpart, const double *__restrict__ Vp,
                                                         const double *__restrict__ Wp, double *__restrict__ coef, int nch)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: row addresses stay scalar
    const int seg = nch * SY_CH;
    if (int(blockIdx.y) >= n_strips) {
        if (blockIdx.x != 0) return;
        __shared__ double red[16];
        const int k = blockIdx.y - n_strips;
        const double *vk = Vp + int64_t(k) * n, *wk = Wp + int64_t(k) * n;
        double sa = 0.0, sb = 0.0;
        for (int c = j + 1 + threadIdx.x; c < n; c += 256) {
            const double vc = v[c];
            sa += wk[c] * vc;
            sb += vk[c] * vc;
        }
        sa = block_sum(sa, red);
        sb = block_sum(sb, red);
        if (threadIdx.x == 0) { coef[2 * k] = sa; coef[2 * k + 1] = sb; }
        return;
    }
    __shared__ double cpart[4][SY_SEG];
    const int strip = (j + 1) / SY_ROWS + blockIdx.y;          // absolute strip: rows 64 strip .. 64 strip + 63
    const int c_first = (strip * SY_ROWS) & ~(SY_CH - 1);      // chunk that holds the strip's first diagonal element
    const int seg0 = c_first + blockIdx.x * seg;
    if (seg0 >= n) return;
    const int a_base = strip * SY_ROWS + wave * SY_WR;
    // Rows outside (j, n) are read from a row inside it and carry no weight: every lane issues the same 16 loads
    // per chunk with no branch between them, so they are all in flight together.
    double racc[SY_WR], va[SY_WR];
    const double *rowp[SY_WR];
#pragma unroll
    for (int q = 0; q < SY_WR; ++q) {
        const int a = a_base + q;
        const bool live = a > j && a < n;
        racc[q] = 0.0;
        va[q] = live ? v[a] : 0.0;
        rowp[q] = A + int64_t(min(max(a, j + 1), n - 1)) * n;
    }
    // one chunk at a time (not unrolled: 16 row loads of 16 bytes per lane are in flight per chunk, more would
    // not fit the register file; requesting the next chunk before summing the current one was tried and costs
    // more in occupancy than it gains); a wavefront parks its column sums in its own LDS row, no barrier until the end
#pragma unroll 1
    for (int ch = 0; ch < nch; ++ch) {
        const int c = seg0 + ch * SY_CH + 2 * lane;
        const int cl = VEC ? min(c, n - 2) : min(c, n - 1);     // a column inside the row for lanes past its end
        const double v0 = (c > j && c < n) ? v[c] : 0.0;
        const double v1 = (c + 1 > j && c + 1 < n) ? v[c + 1] : 0.0;
        double x0[SY_WR], x1[SY_WR];
#pragma unroll
        for (int q = 0; q < SY_WR; ++q) {
            if (VEC) {
                const d2 x = __builtin_nontemporal_load(reinterpret_cast<const d2 *>(rowp[q] + cl));
                x0[q] = x.x; x1[q] = x.y;
            } else {
                x0[q] = __builtin_nontemporal_load(rowp[q] + cl);
                x1[q] = __builtin_nontemporal_load(rowp[q] + min(cl + 1, n - 1));
            }
        }
        double c0 = 0.0, c1 = 0.0;
#pragma unroll
        for (int q = 0; q < SY_WR; ++q) {
            const int a = a_base + q;
            // elements left of the diagonal and past the end of the row count as zero
            const double e0 = (c >= a && c < n) ? x0[q] : 0.0;
            const double e1 = (c + 1 >= a && c + 1 < n) ? x1[q] : 0.0;
            racc[q] += e0 * v0 + e1 * v1;
            c0 += (c > a) ? e0 * va[q] : 0.0;
            c1 += (c + 1 > a) ? e1 * va[q] : 0.0;
        }
        cpart[wave][ch * SY_CH + 2 * lane] = c0;
        cpart[wave][ch * SY_CH + 2 * lane + 1] = c1;
    }
    __syncthreads();
    for (int t = threadIdx.x; t < seg; t += 256)
        if (seg0 + t < n)
            colpart[int64_t(blockIdx.y) * n + seg0 + t] = (cpart[0][t] + cpart[1][t]) + (cpart[2][t] + cpart[3][t]);
#pragma unroll
    for (int q = 0; q < SY_WR; ++q) {
        const int a = a_base + q;
        const double r = wave_sum(racc[q]);
        if (lane == 0 && a > j && a < n) rowpart[int64_t(blockIdx.x) * n + a] = r;
    }
}

// y[c] = sum over the segments of row c's strip of rowpart + sum over the strips up to row c's of colpart
//        - sum_{k<i} (v_k[c] a_k + w_k[c] b_k)          for c > j   (a_k = coef[2k], b_k = coef[2k+1])
__global__ __launch_bounds__(256) void yfix_kernel(int n, int j, int i, const double *__restrict__ rowpart,
                                                   const double *__restrict__ colpart, const double *__restrict__ Vp,
                                                   const double *__restrict__ Wp, const double *__restrict__ coef,
                                                   double *__restrict__ y, int seg)
{
    // seg: columns per segment of the pass that wrote the partial sums
    // 64 columns per workgroup; the strips (up to n / 64 of them) are dealt round-robin to its four wavefronts,
    // four sums in flight each, and met in LDS in a fixed order
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c = j + 1 + blockIdx.x * 64 + lane;
    const int cc = min(c, n - 1);
    const int s_first = (j + 1) / SY_ROWS;
    const int strip = cc / SY_ROWS;
    const int nst = strip - s_first + 1;                  // strips that hold column sums for this column
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    int st = w;
    for (; st + 12 < nst; st += 16) {
        a0 += colpart[int64_t(st) * n + cc];
        a1 += colpart[int64_t(st + 4) * n + cc];
        a2 += colpart[int64_t(st + 8) * n + cc];
        a3 += colpart[int64_t(st + 12) * n + cc];
    }
    for (; st < nst; st += 4) a0 += colpart[int64_t(st) * n + cc];
    part[w][lane] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (w != 0 || c >= n) return;
    double v = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
    const int c_first = (strip * SY_ROWS) & ~(SY_CH - 1);
    const int nseg = (n - c_first + seg - 1) / seg;
    for (int g = 0; g < nseg; ++g) v += rowpart[int64_t(g) * n + c];
    for (int k = 0; k < i; ++k) v -= Vp[int64_t(k) * n + c] * coef[2 * k] + Wp[int64_t(k) * n + c] * coef[2 * k + 1];
    y[c] = v;
}

// y[c] -= sum_{k<i} (v_k[c] a_k + w_k[c] b_k) for c > j, with a_k = coef[2k], b_k = coef[2k+1].
__global__ __launch_bounds__(256) void pfix_kernel(int n, int j, int i, const double *__restrict__ Vp,
                                                   const double *__restrict__ Wp, const double *__restrict__ coef,
                                                   double *__restrict__ y)
{
    const int c = j + 1 + blockIdx.x * 256 + threadIdx.x;
    if (c >= n) return;
    double v = y[c];
    for (int k = 0; k < i; ++k) v -= Vp[int64_t(k) * n + c] * coef[2 * k] + Wp[int64_t(k) * n + c] * coef[2 * k + 1];
    y[c] = v;
}

// One workgroup: w = tau_j y - (tau_j^2 / 2)(y . v) v over columns j+1..
__global__ __launch_bounds__(1024) void w_kernel(int n, int j, const double *__restrict__ tau,
                                                 const double *__restrict__ vc, const double *__restrict__ y,
                                                 double *__restrict__ wc)
{
    __shared__ double red[16];
    const double t = tau[j];
    double dot = 0.0;
    for (int c = j + 1 + threadIdx.x; c < n; c += blockDim.x) dot += y[c] * vc[c];
    dot = block_sum(dot, red);
    const double alpha = 0.5 * t * t * dot;
    for (int c = j + 1 + threadIdx.x; c < n; c += blockDim.x) wc[c] = t * y[c] - alpha * vc[c];
}

// End of a panel of nb columns: A[a, c] -= sum_k (v_k[a] w_k[c] + w_k[a] v_k[c]) for a, c >= jn.
// 64 x 64 tile per workgroup, 4 x 4 elements per thread, the four 64-long slices of the panel in LDS.
// upper_only: tiles strictly below the diagonal are left alone (the upper-triangle pass never reads them).
__global__ __launch_bounds__(256) void syr2k_kernel(double *__restrict__ A, int n, int jn, int nb,
                                                    const double *__restrict__ Vp, const double *__restrict__ Wp,
                                                    int upper_only)
{
    __shared__ double va[NBT][64], wa[NBT][64], vc[NBT][64], wc[NBT][64];
    if (upper_only && blockIdx.y > blockIdx.x) return;
    const int a0 = jn + blockIdx.y * 64, c0 = jn + blockIdx.x * 64;
    for (int e = threadIdx.x; e < NBT * 64; e += 256) {
        const int k = e >> 6, t = e & 63;
        const bool ka = k < nb && a0 + t < n, kc = k < nb && c0 + t < n;
        va[k][t] = ka ? Vp[int64_t(k) * n + a0 + t] : 0.0;
        wa[k][t] = ka ? Wp[int64_t(k) * n + a0 + t] : 0.0;
        vc[k][t] = kc ? Vp[int64_t(k) * n + c0 + t] : 0.0;
        wc[k][t] = kc ? Wp[int64_t(k) * n + c0 + t] : 0.0;
    }
    __syncthreads();
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    double acc[4][4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = 0.0;
#pragma unroll 4
    for (int k = 0; k < NBT; ++k) {
        double av[4], aw[4], cv[4], cw[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            av[p] = va[k][ty * 4 + p];
            aw[p] = wa[k][ty * 4 + p];
            cv[p] = vc[k][tx * 4 + p];
            cw[p] = wc[k][tx * 4 + p];
        }
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[p][q] += av[p] * cw[q] + aw[p] * cv[q];
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int a = a0 + ty * 4 + p;
        if (a >= n) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + tx * 4 + q;
            if (c < n) A[int64_t(a) * n + c] -= acc[p][q];
        }
    }
}

// d_{n-2}, e_{n-2}, d_{n-1} from the 2 x 2 corner once every update has been applied; n >= 2.
__global__ void tri_tail_kernel(const double *__restrict__ A, int n, double *__restrict__ dg, double *__restrict__ e)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int a = n - 2, b = n - 1;
    dg[a] = A[int64_t(a) * n + a];
    e[a] = A[int64_t(a) * n + b];
    dg[b] = A[int64_t(b) * n + b];
    e[b] = 0.0;
}

// ---------------------------------------------------------------- step 1b, accumulation of Q^T

__global__ __launch_bounds__(256) void identity_kernel(double *__restrict__ Zt, int n)
{
    const int64_t total = int64_t(n) * n;
    for (int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x; idx < total; idx += int64_t(gridDim.x) * 256)
        Zt[idx] = (idx / n == idx % n) ? 1.0 : 0.0;
}

// Reflector t of the panel at k0 is row k0+t of A over columns k0+t+1..; anything left of that is zero.
__device__ __forceinline__ double panel_v(const double *__restrict__ A, int n, int k0, int nb, int t, int c)
{
    return (t < nb && c < n && c >= k0 + t + 1) ? A[int64_t(k0 + t) * n + c] : 0.0;
}

// Partial Gram matrices of the panel's reflectors, one per chunk of 128 columns: P[chunk][t][i].
__global__ __launch_bounds__(256) void panel_gram_kernel(const double *__restrict__ A, int n, int k0, int nb,
                                                         double *__restrict__ P)
{
    __shared__ double vs[NB][129];
    const int cbase = k0 + 1 + blockIdx.x * 128;
    for (int e = threadIdx.x; e < NB * 128; e += 256) {
        const int t = e >> 7, c = e & 127;
        vs[t][c] = panel_v(A, n, k0, nb, t, cbase + c);
    }
    __syncthreads();
    const int t = threadIdx.x >> 3, i0 = (threadIdx.x & 7) * 4;
    double g[4] = {0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < 128; ++c) {
        const double vt = vs[t][c];
#pragma unroll
        for (int q = 0; q < 4; ++q) g[q] += vt * vs[i0 + q][c];
    }
    double *out = P + int64_t(blockIdx.x) * NB * NB + t * NB + i0;
#pragma unroll
    for (int q = 0; q < 4; ++q) out[q] = g[q];
}

// T of the compact form H_k0 ... H_{k0+nb-1} = I - V T V^T (upper triangular), from the summed Gram matrix.
__global__ __launch_bounds__(NB * NB) void panel_t_kernel(const double *__restrict__ P, int nchunks, int k0, int nb,
                                                          const double *__restrict__ tau, double *__restrict__ T)
{
    __shared__ double gm[NB][NB + 1], ts[NB][NB + 1];
    {
        // one thread per entry of the Gram matrix, chunks added in order
        const int e = threadIdx.x;
        double s = 0.0;
        for (int ch = 0; ch < nchunks; ++ch) s += P[int64_t(ch) * NB * NB + e];
        gm[e / NB][e % NB] = s;
        ts[e / NB][e % NB] = 0.0;
    }
    __syncthreads();
    for (int i = 0; i < nb; ++i) {
        const double ti = tau[k0 + i];
        const int a = threadIdx.x;
        if (a < i) {
            double s = 0.0;
            for (int t = a; t < i; ++t) s += ts[a][t] * gm[t][i];
            ts[a][i] = -ti * s;
        } else if (a == i) {
            ts[i][i] = ti;
        }
        __syncthreads();
    }
    T[threadIdx.x] = ts[threadIdx.x / NB][threadIdx.x % NB];
}

// Rows r0.. of Zt times the panel: row <- row (I - V T^T V^T), in three kernels so that each streams Zt once with
// tiles large enough to pay for the panel vectors they load:
//   panel_y_kernel       Ypart[ks][r][t] = sum over the ks-th quarter of the columns of Zt[r][c] v_t[c]
//                        (64 rows x 32 reflectors per workgroup, 4 x 2 per thread, 32-column slices through LDS)
//   panel_y2_kernel      Y2[r][t] = sum_{u >= t} (sum_ks Ypart[ks][r][u]) T[t][u]
//   panel_update_kernel  Zt[r][c] -= sum_t Y2[r][t] v_t[c]   (64 x 128 tile per workgroup, 8 x 4 per thread)
constexpr int PA_RB = 64, PA_KS = 4;

__global__ __launch_bounds__(256) void panel_y_kernel(const double *__restrict__ Zt, int n, const double *__restrict__ A,
                                                      int k0, int nb, int r0, int nrows, double *__restrict__ Ypart)
{
    constexpr int CC = 32;
    __shared__ double zs[PA_RB][CC + 1], vs[NB][CC + 1];
    const int rbase = r0 + blockIdx.x * PA_RB;
    const int cfirst = k0 + 1;
    const int nch = (n - cfirst + CC - 1) / CC;
    const int ch0 = int(int64_t(blockIdx.y) * nch / PA_KS), ch1 = int(int64_t(blockIdx.y + 1) * nch / PA_KS);
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;         // rows 4 ty .. 4 ty + 3, reflectors tx and tx + 16
    double acc[4][2] = {{0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}};
    double zreg[8], vreg[4];
    auto fetch = [&](int ch) {
        const int cb = cfirst + ch * CC;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int e = threadIdx.x + q * 256, r = e / CC, c = e % CC;
            zreg[q] = (ch < ch1 && rbase + r < n && cb + c < n) ? Zt[int64_t(rbase + r) * n + cb + c] : 0.0;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = threadIdx.x + q * 256, t = e / CC, c = e % CC;
            vreg[q] = ch < ch1 ? panel_v(A, n, k0, nb, t, cb + c) : 0.0;
        }
    };
    fetch(ch0);
    for (int ch = ch0; ch < ch1; ++ch) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 8; ++q) { const int e = threadIdx.x + q * 256; zs[e / CC][e % CC] = zreg[q]; }
#pragma unroll
        for (int q = 0; q < 4; ++q) { const int e = threadIdx.x + q * 256; vs[e / CC][e % CC] = vreg[q]; }
        __syncthreads();
        fetch(ch + 1);
#pragma unroll 8
        for (int c = 0; c < CC; ++c) {
            const double va = vs[tx][c], vb = vs[tx + 16][c];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const double z = zs[ty * 4 + p][c];
                acc[p][0] += z * va;
                acc[p][1] += z * vb;
            }
        }
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = rbase - r0 + ty * 4 + p;
        if (r < nrows) {
            double *out = Ypart + (int64_t(blockIdx.y) * nrows + r) * NB;
            out[tx] = acc[p][0];
            out[tx + 16] = acc[p][1];
        }
    }
}

__global__ __launch_bounds__(256) void panel_y2_kernel(const double *__restrict__ Ypart, int nrows,
                                                       const double *__restrict__ T, double *__restrict__ Y2)
{
    __shared__ double ts[NB][NB + 1];
    for (int e = threadIdx.x; e < NB * NB; e += 256) ts[e / NB][e % NB] = T[e];
    __syncthreads();
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int r = idx / NB, t = idx % NB;
    if (r >= nrows) return;
    double s = 0.0;
    for (int u = t; u < NB; ++u) {
        double yu = 0.0;
#pragma unroll
        for (int ks = 0; ks < PA_KS; ++ks) yu += Ypart[(int64_t(ks) * nrows + r) * NB + u];
        s += yu * ts[t][u];
    }
    Y2[int64_t(r) * NB + t] = s;
}

__global__ __launch_bounds__(256) void panel_update_kernel(double *__restrict__ Zt, int n, const double *__restrict__ A,
                                                           int k0, int nb, int r0, int nrows, const double *__restrict__ Y2)
{
    constexpr int CT = 128;
    __shared__ __attribute__((aligned(16))) double y2s[PA_RB][NB + 1], vs[NB][CT];
    const int rbase = r0 + blockIdx.x * PA_RB;
    const int cb = k0 + 1 + blockIdx.y * CT;
    for (int e = threadIdx.x; e < PA_RB * NB; e += 256) {
        const int r = e / NB, t = e % NB;
        y2s[r][t] = (rbase - r0 + r < nrows) ? Y2[int64_t(rbase - r0 + r) * NB + t] : 0.0;
    }
    for (int e = threadIdx.x; e < NB * CT; e += 256) {
        const int t = e / CT, c = e % CT;
        vs[t][c] = panel_v(A, n, k0, nb, t, cb + c);
    }
    __syncthreads();
    const int ty = threadIdx.x >> 5, tx = threadIdx.x & 31;         // rows 8 ty .. 8 ty + 7, columns 4 tx .. 4 tx + 3
    double acc[8][4];
#pragma unroll
    for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = 0.0;
#pragma unroll 4
    for (int t = 0; t < NB; ++t) {
        const d2 va = *reinterpret_cast<const d2 *>(&vs[t][tx * 4]);
        const d2 vb = *reinterpret_cast<const d2 *>(&vs[t][tx * 4 + 2]);
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const double y = y2s[ty * 8 + p][t];
            acc[p][0] += y * va.x;
            acc[p][1] += y * va.y;
            acc[p][2] += y * vb.x;
            acc[p][3] += y * vb.y;
        }
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int r = rbase + ty * 8 + p;
        if (r >= n) continue;
        double *row = Zt + int64_t(r) * n;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = cb + tx * 4 + q;
            if (c < n) row[c] -= acc[p][q];
        }
    }
}

// ---------------------------------------------------------------- step 1b, QL rotations

// A batch as the host hands it over: header of 3 * KSW 64-bit integers (lo, hi, off per sweep; sweep s
// rotates i = hi[s] down to lo[s], lo > hi marks an idle stage; its (c, s) pairs start at pairs[off[s]],
// highest index first), then the pairs.
constexpr int ROT_HDR = 3 * KSW;   // in 8-byte words
constexpr int CH = 8;              // time steps per chunk of the rotation pass

// Time-major coefficient table for one pass: tab[t][s] = (c, s) of the rotation stage s applies at
// time t (index rho = top - t + 2 s), the identity where sweep s has none there.
__global__ __launch_bounds__(256) void rot_table_kernel(const long long *__restrict__ hdr,
                                                        const double *__restrict__ pairs, int top, int nsteps,
                                                        double *__restrict__ tab)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= nsteps * KSW) return;
    const int t = idx / KSW, s = idx % KSW;
    const long long lo = hdr[s], hi = hdr[KSW + s], off = hdr[2 * KSW + s];
    const long long rho = (long long)top - t + 2 * s;
    double c = 1.0, sn = 0.0;
    if (rho >= lo && rho <= hi) {
        c = pairs[off + 2 * (hi - rho)];
        sn = pairs[off + 2 * (hi - rho) + 1];
    }
    tab[2 * idx] = c;
    tab[2 * idx + 1] = sn;
}

// One pass of up to KSW sweeps over rows imin..top of Zt.  A workgroup owns 64 columns (one per lane);
// the KSW stages of the pipeline are split over its RW wavefronts, SPW consecutive stages each.  Stage s
// receives row rho = top - t + 2 s at time t, mixes it with the row rho + 1 it holds, and passes that one
// on.  Wave w runs one time step behind wave w - 1 and takes its rows from it through LDS, a chunk of CH
// steps per barrier; wave 0 reads rows from memory, the last wave writes them back.  Rows and
// coefficients of the next chunk are fetched while the current one is computed.
constexpr int RW = 4;
constexpr int SPW = KSW / RW;

__global__ __launch_bounds__(64 * RW) void rot_kernel(double *__restrict__ Zt, int n, int imin, int top, int nchunks,
                                                      const double *__restrict__ tab)
{
    __shared__ double xfer[RW - 1][2][CH][64];
    __shared__ double coef[RW][2][CH * SPW * 2];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int q = blockIdx.x * 64 + lane;
    const bool live = q < n;
    const int qq = live ? q : n - 1;
    double up[SPW], pipe[SPW], cur[CH], nxt[CH];
#pragma unroll
    for (int s = 0; s < SPW; ++s) { up[s] = 0.0; pipe[s] = 0.0; }
    // coefficients of this wave for chunk c: table rows c*CH + w + u (u < CH), its SPW stages' pairs
    const double *ctab = tab + int64_t(w + (lane >> 3)) * (KSW * 2) + w * (SPW * 2) + (lane & 7);
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int rho = top - u;
        cur[u] = (w == 0 && rho >= imin) ? Zt[int64_t(rho) * n + qq] : 0.0;
        nxt[u] = 0.0;
    }
    coef[w][0][lane] = ctab[0];
    __syncthreads();
    const int nticks = nchunks + RW - 1;
    for (int tick = 0; tick < nticks; ++tick) {
        const int ch = tick - w;                       // this wave's chunk in this tick
        if (ch >= 0 && ch < nchunks) {
            const bool more = ch + 1 < nchunks;
            double cfn = 0.0;
            if (more) {
                cfn = ctab[int64_t(ch + 1) * (CH * KSW * 2)];
                if (w == 0) {
#pragma unroll
                    for (int u = 0; u < CH; ++u) {
                        const int rho = top - ((ch + 1) * CH + u);
                        nxt[u] = rho >= imin ? Zt[int64_t(rho) * n + qq] : 0.0;
                    }
                }
            }
            if (w > 0) {
#pragma unroll
                for (int u = 0; u < CH; ++u) cur[u] = xfer[w - 1][ch & 1][u][lane];
            }
            const double *cb = coef[w][ch & 1];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
#pragma unroll
                for (int s = SPW - 1; s >= 0; --s) {
                    const double c = cb[(u * SPW + s) * 2], sn = cb[(u * SPW + s) * 2 + 1];
                    const double in = s == 0 ? cur[u] : pipe[s];
                    const double f = up[s];
                    const double out = sn * in + c * f;        // row rho + 1, done with this sweep
                    up[s] = c * in - sn * f;                   // row rho, kept for the next step
                    if (s == SPW - 1) {
                        if (w == RW - 1) {
                            const int t = ch * CH + u + w;     // time of this step in the whole pipeline
                            const int ro = top - t + 2 * (KSW - 1) + 1;
                            if (live && ro >= imin && ro <= top) Zt[int64_t(ro) * n + q] = out;
                        } else {
                            xfer[w][ch & 1][u][lane] = out;
                        }
                    } else {
                        pipe[s + 1] = out;
                    }
                }
            }
            if (more) {
                coef[w][(ch + 1) & 1][lane] = cfn;
                if (w == 0) {
#pragma unroll
                    for (int u = 0; u < CH; ++u) cur[u] = nxt[u];
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- step 1b, divide and conquer: one merge
//
// The tridiagonal matrix is torn at row m into two halves plus a rank-one term (Cuppen):
//     T = diag(T1', T2') + rho u u^T,   rho = |e_{m-1}|,  u = e_{m-1} + sign(e_{m-1}) e_m,
// T1', T2' being the halves with rho taken off the two diagonal entries next to the tear.  The halves are
// solved by the QL iteration as before (two host threads, rotations applied to their own rows of Zt), which
// leaves Zt = diag(Z1, Z2)^T Q^T and the problem D + rho z z^T with D the eigenvalues of the halves and
// z = diag(Z1, Z2)^T u.  Its eigenpairs are found here, on the device:
//   * z = Zt (Q u), where Q u = row m-1 + sign row m of Q^T is saved before the rotations start;
//   * deflation (host, O(n log n)): components with rho |z_i| below tolerance keep their eigenpair; two close
//     eigenvalues are rotated so that one of them gets a zero component (dc_rot_rows_kernel);
//   * the k remaining eigenvalues are the roots of the secular equation 1 + rho sum_i z_i^2 / (d_i - x) = 0,
//     one per interval between neighbouring d_i: one wavefront per root, measured from the nearer pole so that
//     the differences d_i - x keep full relative accuracy (dc_secular_kernel);
//   * the components are recomputed from the roots (Gu and Eisenstat: zhat_i^2 = prod_j (x_j - d_i) /
//     prod_{j != i} (d_j - d_i)), which makes the eigenvectors u_j = (zhat_i / (d_i - x_j))_i orthogonal to
//     working precision whatever the accuracy of the roots (dc_zhat_kernel, dc_colnorm_kernel, dc_fill_u_kernel);
//   * rows of Zt <- U^T (rows of Zt): a double-precision matrix product (dgemm_tn_kernel).

// uq[c] = Zt[m-1, c] + sgn * Zt[m, c]
__global__ __launch_bounds__(256) void dc_save_u_kernel(const double *__restrict__ Zt, int n, int m, double sgn,
                                                        double *__restrict__ uq)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < n) uq[c] = Zt[int64_t(m - 1) * n + c] + sgn * Zt[int64_t(m) * n + c];
}

// z[r] = Zt[r, :] . uq for rows r0 <= r < r1, one wavefront per row
__global__ __launch_bounds__(256) void dc_gemv_kernel(const double *__restrict__ Zt, int n, int r0, int r1,
                                                      const double *__restrict__ uq, double *__restrict__ z)
{
    const int lane = threadIdx.x & 63;
    const int r = r0 + blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= r1) return;
    const double *row = Zt + int64_t(r) * n;
    double s0 = 0.0, s1 = 0.0;
    int c = lane;
    for (; c + 64 < n; c += 128) { s0 += row[c] * uq[c]; s1 += row[c + 64] * uq[c + 64]; }
    if (c < n) s0 += row[c] * uq[c];
    s0 = wave_sum(s0 + s1);
    if (lane == 0) z[r] = s0;
}

// The deflating rotations, in order: rows a = ra[t], b = rb[t]:  a <- c a + s b,  b <- c b - s a.
// One thread per column; consecutive rotations share a row, so the chain is walked by each thread alone.
__global__ __launch_bounds__(256) void dc_rot_rows_kernel(double *__restrict__ Zt, int n, int nrot,
                                                          const int *__restrict__ ra, const int *__restrict__ rb,
                                                          const double *__restrict__ cs)
{
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= n) return;
    for (int t = 0; t < nrot; ++t) {
        const double c = cs[2 * t], sn = cs[2 * t + 1];
        double *pa = Zt + int64_t(ra[t]) * n + q, *pb = Zt + int64_t(rb[t]) * n + q;
        const double a = *pa, b = *pb;
        *pa = c * a + sn * b;
        *pb = c * b - sn * a;
    }
}

// Root j of 1 + rho sum_i z_i^2 / (d_i - x) = 0 in (d_j, d_{j+1}) (the last one in (d_{k-1}, d_{k-1} + rho |z|^2]),
// d ascending.  One wavefront per root.  x = d_org + mu with org the nearer of the two poles (decided by the
// sign of the function at the midpoint), so f(mu) = R(mu) - a / mu with a = rho z_org^2 and R the sum over the
// other poles, smooth and increasing on the bracket.  Newton steps on f, kept inside a bracket that the sign of
// f narrows every iteration; a step that leaves the bracket is replaced by the fixed point a / R(mu), which
// lands next to a root that hugs its pole, or by the midpoint.
__global__ __launch_bounds__(64) void dc_secular_kernel(int k, const double *__restrict__ d, const double *__restrict__ z,
                                                        double rho, double znorm2, double *__restrict__ mu_out,
                                                        int *__restrict__ org_out)
{
    const int j = blockIdx.x, lane = threadIdx.x;
    const double eps = 2.220446049250313e-16;
    const bool last = j == k - 1;
    const double gap = last ? rho * znorm2 : d[j + 1] - d[j];
    // value, derivative and magnitude of f at mu measured from pole `org`
    auto eval = [&](int org, double mu, double &f, double &fp, double &mag, double &R) {
        const double dorg = d[org];
        double sr = 0.0, sp = 0.0, sm = 0.0;
        for (int i = lane; i < k; i += 64) {
            if (i == org) continue;
            const double zi = z[i];
            const double t = zi / ((d[i] - dorg) - mu);
            const double term = zi * t;
            sr += term;
            sp += t * t;
            sm += fabs(term);
        }
        sr = wave_sum(sr); sp = wave_sum(sp); sm = wave_sum(sm);
        const double a = rho * z[org] * z[org];
        R = 1.0 + rho * sr;
        f = R - a / mu;
        fp = rho * sp + a / (mu * mu);
        mag = 1.0 + rho * sm + fabs(a / mu);
    };
    int org = j;
    double lo = 0.0, hi = last ? gap : 0.5 * gap;      // f(lo+) = -inf, f(hi) >= 0 when the root lies in the left half
    double f, fp, mag, R;
    if (!last) {
        eval(j, 0.5 * gap, f, fp, mag, R);
        if (f < 0.0) { org = j + 1; lo = -0.5 * gap; hi = 0.0; }    // root in the right half: measure from d_{j+1}
    }
    const double a = rho * z[org] * z[org];
    double mu = 0.5 * (lo + hi);
    for (int it = 0; it < 400; ++it) {
        eval(org, mu, f, fp, mag, R);
        if (fabs(f) <= 8.0 * eps * mag) break;
        if (f > 0.0) hi = mu; else lo = mu;
        if (hi - lo <= 2.0 * eps * fmax(fabs(lo), fabs(hi))) { mu = (f > 0.0) ? lo + 0.5 * (hi - lo) : mu; break; }
        double next = mu - f / fp;
        if (!(next > lo && next < hi)) {
            const double fix = a / R;                    // root of R(mu) - a / x = 0 with R frozen
            next = (fix > lo && fix < hi) ? fix : 0.5 * (lo + hi);
        }
        if (next == mu) break;
        mu = next;
    }
    if (lane == 0) { mu_out[j] = mu; org_out[j] = org; }
}

// d_i - x_j with x_j = d[org_j] + mu_j
__device__ __forceinline__ double dc_delta(const double *__restrict__ d, const double *__restrict__ mu,
                                           const int *__restrict__ org, int i, int j)
{
    return (d[i] - d[org[j]]) - mu[j];
}

// zhat_i = sign(z_i) sqrt(| (d_i - x_i) prod_{j != i} (d_i - x_j) / (d_i - d_j) |); one wavefront per i, each lane a
// contiguous run of j so that neighbouring ratios (which interlace) meet in the same partial product.
__global__ __launch_bounds__(64) void dc_zhat_kernel(int k, const double *__restrict__ d, const double *__restrict__ z,
                                                     const double *__restrict__ mu, const int *__restrict__ org,
                                                     double *__restrict__ zhat)
{
    const int i = blockIdx.x, lane = threadIdx.x;
    const int per = (k + 63) / 64;
    const int j0 = lane * per, j1 = min(k, j0 + per);
    double prod = 1.0;
    for (int j = j0; j < j1; ++j) {
        const double num = dc_delta(d, mu, org, i, j);
        prod *= (j == i) ? num : num / (d[i] - d[j]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) prod *= __shfl_xor(prod, off, 64);
    if (lane == 0) zhat[i] = copysign(sqrt(fabs(prod)), z[i]);
}

// 1 / || (zhat_i / (d_i - x_j))_i ||, one wavefront per j
__global__ __launch_bounds__(64) void dc_colnorm_kernel(int k, const double *__restrict__ d, const double *__restrict__ zhat,
                                                        const double *__restrict__ mu, const int *__restrict__ org,
                                                        double *__restrict__ inv_norm)
{
    const int j = blockIdx.x, lane = threadIdx.x;
    double s = 0.0;
    for (int i = lane; i < k; i += 64) {
        const double v = zhat[i] / dc_delta(d, mu, org, i, j);
        s += v * v;
    }
    s = wave_sum(s);
    if (lane == 0) inv_norm[j] = 1.0 / sqrt(s);
}

// U[i, j] = zhat_i / (d_i - x_j) / norm_j, row-major k x k
__global__ __launch_bounds__(256) void dc_fill_u_kernel(int k, const double *__restrict__ d, const double *__restrict__ zhat,
                                                        const double *__restrict__ mu, const int *__restrict__ org,
                                                        const double *__restrict__ inv_norm, double *__restrict__ U)
{
    const int j = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
    if (j < k) U[int64_t(i) * k + j] = zhat[i] / dc_delta(d, mu, org, i, j) * inv_norm[j];
}

// T[i, :] = Zt[rows[i], :]
__global__ __launch_bounds__(256) void dc_gather_kernel(const double *__restrict__ Zt, int n, const int *__restrict__ rows,
                                                        double *__restrict__ T)
{
    const int i = blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
    if (c < n) T[int64_t(i) * n + c] = Zt[int64_t(rows[i]) * n + c];
}

// Zt[rows[j], c] = sum_i U[i, j] T[i, c]  (j < k, c < n, i < k): C = U^T T in double precision.  The contraction
// index is the row index of both operands, so a slice of 8 rows of U and of T is two sets of contiguous runs:
// 128 x 128 tile per workgroup, 8 x 8 per thread as 2-wide pieces 32 apart (conflict-free 16-byte LDS reads),
// next slice fetched into registers while the current one is multiplied from LDS.
__global__ __launch_bounds__(256) void dgemm_tn_kernel(const double *__restrict__ U, int k, const double *__restrict__ T,
                                                       int n, const int *__restrict__ rows, double *__restrict__ Zt)
{
    constexpr int BT = 128, BK = 8;
    __shared__ __attribute__((aligned(16))) double As[BK][BT], Bs[BK][BT];
    const int j0 = blockIdx.y * BT, c0 = blockIdx.x * BT;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    // loader: thread -> (slice row lr, 4 consecutive columns lc)
    const int lr = threadIdx.x >> 5, lc = (threadIdx.x & 31) * 4;
    double acc[8][8];
#pragma unroll
    for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[p][q] = 0.0;
    double ra[4], rb[4];
    auto fetch = [&](int i0) {
        const int i = i0 + lr;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            ra[e] = (i < k && j0 + lc + e < k) ? U[int64_t(i) * k + j0 + lc + e] : 0.0;
            rb[e] = (i < k && c0 + lc + e < n) ? T[int64_t(i) * n + c0 + lc + e] : 0.0;
        }
    };
    fetch(0);
    for (int i0 = 0; i0 < k; i0 += BK) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) { As[lr][lc + e] = ra[e]; Bs[lr][lc + e] = rb[e]; }
        __syncthreads();
        if (i0 + BK < k) fetch(i0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            double a[8], b[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const d2 av = *reinterpret_cast<const d2 *>(&As[kk][q * 32 + ty * 2]);
                const d2 bv = *reinterpret_cast<const d2 *>(&Bs[kk][q * 32 + tx * 2]);
                a[2 * q] = av.x; a[2 * q + 1] = av.y;
                b[2 * q] = bv.x; b[2 * q + 1] = bv.y;
            }
#pragma unroll
            for (int p = 0; p < 8; ++p)
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[p][q] += a[p] * b[q];
        }
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int j = j0 + (p >> 1) * 32 + ty * 2 + (p & 1);
        if (j >= k) continue;
        double *out = Zt + int64_t(rows[j]) * n;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int c = c0 + (q >> 1) * 32 + tx * 2 + (q & 1);
            if (c < n) out[c] = acc[p][q];
        }
    }
}

// ---------------------------------------------------------------- step 1c

// Row j of W from eigenvector row ord[j] of Zt: scaled by 1/sqrt(lambda), sign chosen so that the entry
// of largest magnitude (the first of them) is positive; rows from r on are zero.
__global__ __launch_bounds__(256) void finish_kernel(const double *__restrict__ Zt, int n, const int *__restrict__ ord,
                                                     const double *__restrict__ lam, int r, float *__restrict__ W,
                                                     int64_t ldw)
{
    __shared__ double bestv[256];
    __shared__ int besti[256];
    const int j = blockIdx.x;
    float *wr = W + int64_t(j) * ldw;
    if (j >= r) {
        for (int k = threadIdx.x; k < n; k += 256) wr[k] = 0.f;
        return;
    }
    const double *u = Zt + int64_t(ord[j]) * n;
    double bv = -1.0;
    int bi = n;
    for (int k = threadIdx.x; k < n; k += 256) {
        const double a = fabs(u[k]);
        if (a > bv) { bv = a; bi = k; }
    }
    bestv[threadIdx.x] = bv;
    besti[threadIdx.x] = bi;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (int(threadIdx.x) < off) {
            const double ov = bestv[threadIdx.x + off];
            const int oi = besti[threadIdx.x + off];
            if (ov > bestv[threadIdx.x] || (ov == bestv[threadIdx.x] && oi < besti[threadIdx.x])) {
                bestv[threadIdx.x] = ov;
                besti[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    const double sgn = u[besti[0]] < 0.0 ? -1.0 : 1.0;
    const double scale = sgn / sqrt(lam[j]);
    for (int k = threadIdx.x; k < n; k += 256) wr[k] = float(scale * u[k]);
}

// ---------------------------------------------------------------- host side

struct DevCarve {
    size_t off_A, off_Zt, off_vec, off_panel, off_P, off_T, off_cs, off_tab, off_ord, off_lam, bytes;
    size_t off_cs2, off_tab2, off_G, off_dc, off_uq;   // further QL instances, gathered rows, vectors of the merges
    size_t off_rowpart, off_colpart;                   // partial sums of the upper-triangle pass
    size_t off_Y;                                      // Y parts and Y2 of the reflector accumulation
    size_t cs_doubles;     // capacity of ONE of the rotation buffers, header included
    size_t cs_bytes, tab_bytes;
};

constexpr int kDcMin = 512;      // matrices from this size on are torn apart and merged on the device
constexpr int kMaxLeaves = 8;    // pieces the tridiagonal problem is torn into at most
std::atomic<int> g_dc_enabled{1};
std::atomic<int> g_upper_pass{1};   // 1: the reduction reads and maintains the upper triangle only

// Depth of the tearing: 2^levels leaves.
inline int dc_levels(int64_t n) { return n >= 8192 ? 3 : n >= 2048 ? 2 : n >= kDcMin ? 1 : 0; }

DevCarve dev_carve(int64_t n)
{
    DevCarve c;
    const size_t nn = round_up(size_t(n) * size_t(n) * 8, kAlign);
    const size_t vec = round_up(size_t(n) * 8, kAlign);
    size_t o = 0;
    c.off_A = o; o += nn;
    c.off_Zt = o; o += nn;
    c.off_vec = o; o += 8 * vec;                   // x, y, coef, dg, e, tau (two spare)
    c.off_panel = o; o += 2 * round_up(size_t(NBT) * size_t(n) * 8, kAlign);   // panel vectors v_k, w_k
    const size_t nchunks = size_t(n) / 128 + 2;
    c.off_P = o; o += round_up(nchunks * NB * NB * 8, kAlign);
    c.off_T = o; o += round_up(size_t(NB) * NB * 8, kAlign);
    c.cs_doubles = ROT_HDR + size_t(KSW) * 2 * size_t(std::max<int64_t>(n, 1));
    c.cs_bytes = round_up(c.cs_doubles * 8, kAlign);
    c.off_cs = o; o += 2 * c.cs_bytes;
    c.tab_bytes = round_up((size_t(n) + 2 * KSW + 2 * CH) * KSW * 2 * 8, kAlign);
    c.off_tab = o; o += c.tab_bytes;
    c.off_ord = o; o += round_up(size_t(n) * 4, kAlign);
    c.off_lam = o; o += vec;
    // divide and conquer (n >= kDcMin): buffers of the further QL instances, the gathered rows of Zt (n x n),
    // fourteen vectors (z, d, z kept, mu, zhat, 1/norm, rotation pairs (2), origin, rows, rotation rows (2), spare)
    // and one saved vector Q u per tear
    const size_t extra = size_t((1 << dc_levels(n)) - 1);
    c.off_cs2 = o; o += extra * 2 * c.cs_bytes;
    c.off_tab2 = o; o += extra * c.tab_bytes;
    c.off_G = o; o += n >= kDcMin ? nn : 0;
    c.off_dc = o; o += 14 * vec;
    c.off_uq = o; o += extra * vec;
    // segments per row: n / 512 of the long ones, or, once the trailing matrix has SY_SMALL rows or fewer (its first
    // chunk then starts no more than SY_SMALL + SY_CH columns from the end), that many columns in short ones
    c.off_rowpart = o;
    o += (std::max(size_t(n) / SY_SEG, std::min(size_t(n), size_t(SY_SMALL + SY_CH)) / (SY_NCH_SMALL * SY_CH)) + 2) * vec;
    c.off_colpart = o; o += (size_t(n) / SY_ROWS + 2) * vec;
    c.off_Y = o; o += round_up(size_t(5) * size_t(std::max<int64_t>(n, 1)) * 32 * 8, kAlign);
    c.bytes = o;
    return c;
}

bool verbose()
{
    const char *v = std::getenv("LPD_VERBOSE");
    return v && v[0] == '1';
}

#define LPD_HIP(call)                                             \
    do {                                                          \
        if ((call) != hipSuccess) { status = LPD_ERR_HIP; goto done; } \
    } while (0)

// Page-locked staging and events of lpd_whiten: made at its first call (and when a larger matrix comes
// along), kept until the process ends, so that repeated calls (one per kernel parameter of a grid search)
// allocate nothing.  One call at a time uses it: lpd_whiten holds `mu` while it runs.
struct Staging {
    std::mutex mu;
    int64_t n_cap = 0;
    size_t cs_doubles = 0;
    double *cs_h[2 * kMaxLeaves] = {};        // rotation batches: two per QL instance
    hipEvent_t cs_free[2 * kMaxLeaves] = {};
    hipEvent_t tri_done = nullptr;
    double *dge_h = nullptr;                                  // 3 n doubles: tridiagonal matrix; order and eigenvalues
    double *dc_h = nullptr;                                   // 8 n doubles: vectors of the merge
    bool reserve(int64_t n, size_t cs_d)
    {
        if (n <= n_cap) return true;
        for (int b = 0; b < 2 * kMaxLeaves; ++b) if (cs_h[b]) { (void)hipHostFree(cs_h[b]); cs_h[b] = nullptr; }
        if (dge_h) { (void)hipHostFree(dge_h); dge_h = nullptr; }
        if (dc_h) { (void)hipHostFree(dc_h); dc_h = nullptr; }
        n_cap = 0;
        for (int b = 0; b < 2 * (1 << dc_levels(n)); ++b)
            if (hipHostMalloc(reinterpret_cast<void **>(&cs_h[b]), cs_d * 8, hipHostMallocDefault) != hipSuccess) return false;
        if (hipHostMalloc(reinterpret_cast<void **>(&dge_h), size_t(n) * 8 * 3, hipHostMallocDefault) != hipSuccess) return false;
        if (hipHostMalloc(reinterpret_cast<void **>(&dc_h), size_t(n) * 8 * 8, hipHostMallocDefault) != hipSuccess) return false;
        for (int b = 0; b < 2 * kMaxLeaves; ++b)
            if (!cs_free[b] && hipEventCreateWithFlags(&cs_free[b], hipEventDisableTiming) != hipSuccess) return false;
        if (!tri_done && hipEventCreateWithFlags(&tri_done, hipEventDisableTiming) != hipSuccess) return false;
        n_cap = n;
        cs_doubles = cs_d;
        return true;
    }
};
Staging g_staging;

// One QL iteration on rows row0 .. row0 + sz - 1 of the tridiagonal problem: the host finds the rotations,
// the device applies them to those rows of Zt, 16 sweeps per pass, two batches in flight.
struct QlRun {
    int n = 0, row0 = 0, sz = 0;
    double *Zt = nullptr;
    hipStream_t s = nullptr;
    double *cs_h[2] = {nullptr, nullptr};
    hipEvent_t cs_free[2] = {nullptr, nullptr};
    double *cs_d[2] = {nullptr, nullptr};
    double *tab_d = nullptr;
    size_t cs_doubles = 0;
    int device = 0;
    bool talk = false;
    int64_t nbatch = 0;
    int hip_fail = 0;        // 1: a HIP call failed, 2: a batch did not fit what it was promised
    bool ok = false;

    void run(double *dg, double *e)
    {
        if (hipSetDevice(device) != hipSuccess) { hip_fail = 1; return; }
        // the QL iteration writes its rotations straight into the page-locked buffer of the batch, behind
        // the header; the buffer is free once the copy queued from it two batches ago has run
        auto buffer = [&]() -> double * {
            const int b = int(nbatch & 1);
            if (hip_fail || hipEventSynchronize(cs_free[b]) != hipSuccess) { hip_fail = hip_fail ? hip_fail : 1; return nullptr; }
            return cs_h[b] + ROT_HDR;
        };
        auto apply = [&](const std::vector<lpd_host::Sweep> &sw, const double *cs, size_t ncs) {
            if (hip_fail || sw.empty()) return;
            const int b = int(nbatch & 1);
            ++nbatch;
            long long *hdr = reinterpret_cast<long long *>(cs_h[b]);
            int imin = sz, imax = 0;
            if (cs != cs_h[b] + ROT_HDR) { hip_fail = 2; return; }
            for (int k = 0; k < KSW; ++k) { hdr[k] = 1; hdr[KSW + k] = 0; hdr[2 * KSW + k] = 0; }
            for (size_t k = 0; k < sw.size() && k < size_t(KSW); ++k) {
                hdr[k] = sw[k].lo + row0;
                hdr[KSW + k] = sw[k].hi + row0;
                hdr[2 * KSW + k] = (long long)sw[k].off;
                imin = std::min(imin, int(sw[k].lo));
                imax = std::max(imax, int(sw[k].hi));
            }
            if (ROT_HDR + ncs > cs_doubles || sw.size() > size_t(KSW) || imax + 1 >= sz || imin < 0 || imin > imax) {
                hip_fail = 2;
                return;
            }
            if (hipMemcpyAsync(cs_d[b], cs_h[b], (ROT_HDR + ncs) * 8, hipMemcpyHostToDevice, s) != hipSuccess ||
                hipEventRecord(cs_free[b], s) != hipSuccess) { hip_fail = 1; return; }
            const int top = imax + 1 + row0, bottom = imin + row0;
            const int nsteps = (top - bottom) + 2 * KSW;            // t = 0 .. t_last
            const int nchunks = (nsteps + CH - 1) / CH;
            const int tab_steps = (nchunks + 1) * CH;               // the later waves read RW - 1 steps further
            hipLaunchKernelGGL(rot_table_kernel, dim3((tab_steps * KSW + 255) / 256), dim3(256), 0, s,
                               reinterpret_cast<const long long *>(cs_d[b]), cs_d[b] + ROT_HDR, top, tab_steps, tab_d);
            hipLaunchKernelGGL(rot_kernel, dim3((n + 63) / 64), dim3(64 * RW), 0, s, Zt, n, bottom, top, nchunks, tab_d);
            if (hipGetLastError() != hipSuccess) hip_fail = 1;
        };
        int last_decile = -1;
        auto prog = [&](int64_t l) {
            const int dec = int(l * 10 / std::max(sz, 1));
            if (talk && dec != last_decile) {
                last_decile = dec;
                std::fprintf(stderr, "[lpd_whiten B=%d] QL iteration on rows %d..%d: %d%%\n", n, row0, row0 + sz - 1, dec * 10);
                std::fflush(stderr);
            }
        };
        ok = lpd_host::tridiag_ql(dg, e, sz, KSW, buffer, apply, prog);
    }
};

// Pointers into the workspace that the merge uses.
struct DcBuffers {
    double *Zt, *U, *G;                 // n x n each; U overlays the matrix that held the reflectors
    double *z, *dk, *zk, *mu, *zhat, *inv_norm, *rotcs;
    int *org, *rows, *ra, *rb;
};

// One tear of the tridiagonal matrix: rows r0 .. r0 + sz - 1 fall into [r0, m) and [m, r0 + sz).
struct Tear { int r0, sz, m; double rho, sgn; double *uq; };

// The merge of the two solved halves of a tear (see the kernels above).  dg: eigenvalues by row of Zt, those of
// the halves on entry, those of the block on exit.  stage: 8 n doubles of page-locked memory.
int dc_merge(int n, const Tear &tr, std::vector<double> &dg, const DcBuffers &b, double *stage, hipStream_t s, bool talk)
{
    const int r0 = tr.r0, r1 = tr.r0 + tr.sz;
    double rho = tr.rho;
    const double eps = 2.220446049250313e-16;
    double *z_h = stage, *dk_h = stage + n, *zk_h = stage + 2 * size_t(n), *rot_h = stage + 3 * size_t(n),
           *mu_h = stage + 5 * size_t(n);
    int *rows_h = reinterpret_cast<int *>(stage + 6 * size_t(n)), *ra_h = rows_h + n, *rb_h = ra_h + n, *org_h = rb_h + n;

    hipLaunchKernelGGL(dc_gemv_kernel, dim3((tr.sz + 3) / 4), dim3(256), 0, s, b.Zt, n, r0, r1, tr.uq, b.z);
    if (hipGetLastError() != hipSuccess ||
        hipMemcpyAsync(z_h + r0, b.z + r0, size_t(tr.sz) * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return LPD_ERR_HIP;

    // z has norm sqrt(2) (one unit row of each half): scale it to 1 and rho with it
    double zz = 0.0;
    for (int i = r0; i < r1; ++i) zz += z_h[i] * z_h[i];
    if (!(zz > 0.0) || !std::isfinite(zz)) return LPD_ERR_NUMERIC;
    const double zs = 1.0 / std::sqrt(zz);
    for (int i = r0; i < r1; ++i) z_h[i] *= zs;
    rho *= zz;

    double dmax = 0.0, zmax = 0.0;
    for (int i = r0; i < r1; ++i) { dmax = std::max(dmax, std::fabs(dg[size_t(i)])); zmax = std::max(zmax, std::fabs(z_h[i])); }
    const double tol = 8.0 * eps * std::max(dmax, zmax);
    if (rho * zmax <= tol) return LPD_OK;           // the halves do not see each other: nothing to merge

    std::vector<int> perm(size_t(tr.sz), 0);
    std::iota(perm.begin(), perm.end(), r0);
    std::stable_sort(perm.begin(), perm.end(), [&](int a, int c) { return dg[size_t(a)] < dg[size_t(c)]; });
    int k = 0, nrot = 0, pj = -1;
    for (int idx = 0; idx < tr.sz; ++idx) {
        const int i = perm[size_t(idx)];
        if (rho * std::fabs(z_h[i]) <= tol) continue;        // its eigenpair stands as it is
        if (pj < 0) { pj = i; continue; }
        double sn = z_h[pj], c = z_h[i];
        const double tau = std::hypot(c, sn);
        const double t = dg[size_t(i)] - dg[size_t(pj)];
        c /= tau;
        sn = -sn / tau;
        if (std::fabs(t * c * sn) <= tol) {
            // two eigenvalues too close to tell apart: rotate their vectors so that pj carries no component
            z_h[i] = tau;
            z_h[pj] = 0.0;
            ra_h[nrot] = pj; rb_h[nrot] = i;
            rot_h[2 * nrot] = c; rot_h[2 * nrot + 1] = sn;
            ++nrot;
            const double dp = dg[size_t(pj)], di = dg[size_t(i)];
            dg[size_t(pj)] = dp * c * c + di * sn * sn;
            dg[size_t(i)] = dp * sn * sn + di * c * c;
        } else {
            rows_h[k++] = pj;
        }
        pj = i;
    }
    if (pj >= 0) rows_h[k++] = pj;
    double zn2 = 0.0;
    for (int i = 0; i < k; ++i) { dk_h[i] = dg[size_t(rows_h[i])]; zk_h[i] = z_h[rows_h[i]]; zn2 += zk_h[i] * zk_h[i]; }
    for (int i = 1; i < k; ++i)
        if (!(dk_h[i] > dk_h[i - 1])) return LPD_ERR_NUMERIC;    // cannot happen: equal values deflate
    if (talk) {
        std::fprintf(stderr, "[lpd_whiten B=%d] merge of rows %d..%d: %d of %d eigenvalues from the secular equation, "
                     "%d deflating rotations\n", n, r0, r1 - 1, k, tr.sz, nrot);
        std::fflush(stderr);
    }
    if (k == 0) return LPD_OK;

    if (hipMemcpyAsync(b.dk, dk_h, size_t(k) * 8, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(b.zk, zk_h, size_t(k) * 8, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(b.rows, rows_h, size_t(k) * 4, hipMemcpyHostToDevice, s) != hipSuccess)
        return LPD_ERR_HIP;
    if (nrot > 0) {
        if (hipMemcpyAsync(b.ra, ra_h, size_t(nrot) * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(b.rb, rb_h, size_t(nrot) * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(b.rotcs, rot_h, size_t(nrot) * 16, hipMemcpyHostToDevice, s) != hipSuccess)
            return LPD_ERR_HIP;
        hipLaunchKernelGGL(dc_rot_rows_kernel, dim3((n + 255) / 256), dim3(256), 0, s, b.Zt, n, nrot, b.ra, b.rb, b.rotcs);
    }
    hipLaunchKernelGGL(dc_secular_kernel, dim3(k), dim3(64), 0, s, k, b.dk, b.zk, rho, zn2, b.mu, b.org);
    hipLaunchKernelGGL(dc_zhat_kernel, dim3(k), dim3(64), 0, s, k, b.dk, b.zk, b.mu, b.org, b.zhat);
    hipLaunchKernelGGL(dc_colnorm_kernel, dim3(k), dim3(64), 0, s, k, b.dk, b.zhat, b.mu, b.org, b.inv_norm);
    hipLaunchKernelGGL(dc_fill_u_kernel, dim3((k + 255) / 256, k), dim3(256), 0, s, k, b.dk, b.zhat, b.mu, b.org,
                       b.inv_norm, b.U);
    hipLaunchKernelGGL(dc_gather_kernel, dim3((n + 255) / 256, k), dim3(256), 0, s, b.Zt, n, b.rows, b.G);
    hipLaunchKernelGGL(dgemm_tn_kernel, dim3((n + 127) / 128, (k + 127) / 128), dim3(256), 0, s, b.U, k, b.G, n, b.rows, b.Zt);
    if (hipGetLastError() != hipSuccess ||
        hipMemcpyAsync(mu_h, b.mu, size_t(k) * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(org_h, b.org, size_t(k) * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return LPD_ERR_HIP;
    for (int j = 0; j < k; ++j) {
        const double lam = dk_h[org_h[j]] + mu_h[j];
        if (!std::isfinite(lam)) return LPD_ERR_NUMERIC;
        dg[size_t(rows_h[j])] = lam;
    }
    return LPD_OK;
}

}  // namespace

void lpd_host::set_divide_and_conquer(int on) { g_dc_enabled.store(on ? 1 : 0, std::memory_order_relaxed); }
void lpd_host::set_upper_triangle_pass(int on) { g_upper_pass.store(on ? 1 : 0, std::memory_order_relaxed); }

extern "C" int lpd_whiten_workspace(int64_t B, size_t *bytes)
{
    if (!bytes) return LPD_ERR_NULL;
    if (B < 0 || B > 46340) return LPD_ERR_SHAPE;     // B * B must fit 32-bit row arithmetic
    *bytes = dev_carve(B).bytes;
    return LPD_OK;
}

extern "C" int lpd_whiten(const float *L, int64_t B, int64_t d, int64_t ldl, double gamma, double clip_ratio, float *W,
                          int64_t ldw, double *eig_host, int64_t *rank, void *workspace, size_t workspace_bytes,
                          void *hip_stream, double *phase_seconds)
{
    if (B < 0 || d < 0 || B > 46340 || d > (int64_t(1) << 24)) return LPD_ERR_SHAPE;
    if (!rank) return LPD_ERR_NULL;
    *rank = 0;
    if (B == 0) return LPD_OK;
    if (!W || (d > 0 && !L)) return LPD_ERR_NULL;
    if (ldw < B || (d > 0 && ldl < d)) return LPD_ERR_LD;
    const int n = int(B);
    const DevCarve cv = dev_carve(n);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < cv.bytes)
        return LPD_ERR_WORKSPACE;

    int status = LPD_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    double *A = reinterpret_cast<double *>(ws + cv.off_A);
    double *Zt = reinterpret_cast<double *>(ws + cv.off_Zt);
    const size_t vec = round_up(size_t(n) * 8, kAlign);
    auto vecp = [&](int k) { return reinterpret_cast<double *>(ws + cv.off_vec + size_t(k) * vec); };
    double *xrow = vecp(0), *coef = vecp(1);
    double *y = vecp(4), *dg_d = vecp(5), *e_d = vecp(6), *tau_d = vecp(7);
    double *Vp = reinterpret_cast<double *>(ws + cv.off_panel);
    double *Wp = reinterpret_cast<double *>(ws + cv.off_panel + round_up(size_t(NBT) * size_t(n) * 8, kAlign));
    double *P = reinterpret_cast<double *>(ws + cv.off_P);
    double *T = reinterpret_cast<double *>(ws + cv.off_T);
    double *cs_d[2] = {reinterpret_cast<double *>(ws + cv.off_cs),
                       reinterpret_cast<double *>(ws + cv.off_cs + round_up(cv.cs_doubles * 8, kAlign))};
    double *tab_d = reinterpret_cast<double *>(ws + cv.off_tab);
    int *ord_d = reinterpret_cast<int *>(ws + cv.off_ord);
    double *lam_d = reinterpret_cast<double *>(ws + cv.off_lam);

    // Phase timing (phase_seconds given, or LPD_VERBOSE=1 for lines on stderr): the stream is drained at
    // each phase boundary, which costs the overlap of the reflector accumulation with the host's QL start.
    const bool talk = verbose();
    const auto t_start = std::chrono::steady_clock::now();
    int phase = -1;
    double t_phase = 0.0;
    auto say = [&](const char *what) {
        if (!talk && !phase_seconds) return;
        (void)hipStreamSynchronize(s);
        const double sec = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count();
        if (phase_seconds && phase >= 0 && phase < 5) phase_seconds[phase] = sec - t_phase;
        ++phase;
        t_phase = sec;
        if (talk) { std::fprintf(stderr, "[lpd_whiten B=%d] +%.3f s: %s\n", n, sec, what); std::fflush(stderr); }
    };
    if (phase_seconds)
        for (int k = 0; k < 5; ++k) phase_seconds[k] = 0.0;

    // page-locked staging (rotation batches, the tridiagonal matrix, order and eigenvalues, the vectors of the
    // merge) and events: the process-wide set, made at the first call; held for the duration of this one
    std::lock_guard<std::mutex> staging_lock(g_staging.mu);
    double *dge_h = nullptr;
    hipEvent_t tri_done = nullptr;
    std::vector<double> dg(size_t(n), 0.0), e(size_t(n), 0.0);
    std::vector<int64_t> ord;
    std::vector<Tear> tears;                  // children before parents
    std::vector<std::pair<int, int>> leaves;  // (first row, rows)
    QlRun ql[kMaxLeaves];
    int device = 0;
    int64_t r = 0;
    const int levels = g_dc_enabled.load(std::memory_order_relaxed) != 0 ? dc_levels(n) : 0;
    const int nleaves = 1 << levels;

    if (!g_staging.reserve(n, cv.cs_doubles)) { status = LPD_ERR_HIP; goto done; }
    dge_h = g_staging.dge_h;
    tri_done = g_staging.tri_done;
    LPD_HIP(hipGetDevice(&device));
    for (int q = 0; q < nleaves; ++q) {
        ql[q].n = n; ql[q].Zt = Zt; ql[q].s = s; ql[q].device = device; ql[q].talk = talk;
        ql[q].cs_doubles = cv.cs_doubles;
        for (int b = 0; b < 2; ++b) {
            // an event that was never recorded counts as complete; one left over from an earlier call has long run
            ql[q].cs_h[b] = g_staging.cs_h[2 * q + b];
            ql[q].cs_free[b] = g_staging.cs_free[2 * q + b];
            ql[q].cs_d[b] = reinterpret_cast<double *>(
                ws + (q == 0 ? cv.off_cs + size_t(b) * cv.cs_bytes : cv.off_cs2 + size_t(2 * (q - 1) + b) * cv.cs_bytes));
        }
        ql[q].tab_d = reinterpret_cast<double *>(ws + (q == 0 ? cv.off_tab : cv.off_tab2 + size_t(q - 1) * cv.tab_bytes));
    }

    say("landmark kernel matrix");
    {
        const dim3 grid((n + 15) / 16, (n + 15) / 16);
        hipLaunchKernelGGL(kll_kernel, grid, dim3(256), 0, s, L, n, int(d), ldl, gamma, A);
        LPD_HIP(hipGetLastError());
    }

    say("tridiagonalisation");
    {
        const bool even = n % 2 == 0;
        const bool upper = g_upper_pass.load(std::memory_order_relaxed) != 0;
        double *rowpart = reinterpret_cast<double *>(ws + cv.off_rowpart);
        double *colpart = reinterpret_cast<double *>(ws + cv.off_colpart);
        for (int j0 = 0; j0 + 2 < n; j0 += NBT) {
            const int nb = std::min(NBT, n - 2 - j0);
            for (int i = 0; i < nb; ++i) {
                const int j = j0 + i;
                double *vi = Vp + int64_t(i) * n, *wi = Wp + int64_t(i) * n;
                hipLaunchKernelGGL(rowfix_kernel, dim3((n - j + 255) / 256), dim3(256), 0, s, A, n, j, i, Vp, Wp, xrow);
                hipLaunchKernelGGL(hh_kernel, dim3(1), dim3(1024), 0, s, A, n, j, xrow, vi, dg_d, e_d, tau_d);
                const int rows = n - j - 1;
                if (upper) {
                    const int s_first = (j + 1) / SY_ROWS;
                    const int n_strips = (n - 1) / SY_ROWS - s_first + 1;
                    const int c_first = (s_first * SY_ROWS) & ~(SY_CH - 1);
                    const int nch = rows <= SY_SMALL ? SY_NCH_SMALL : SY_NCH;
                    const int seg = nch * SY_CH;
                    const int nseg = (n - c_first + seg - 1) / seg;
                    if (even)
                        hipLaunchKernelGGL((symv_upper_kernel<true>), dim3(nseg, n_strips + i), dim3(256), 0, s, A, n, j,
                                           n_strips, vi, rowpart, colpart, Vp, Wp, coef, nch);
                    else
                        hipLaunchKernelGGL((symv_upper_kernel<false>), dim3(nseg, n_strips + i), dim3(256), 0, s, A, n, j,
                                           n_strips, vi, rowpart, colpart, Vp, Wp, coef, nch);
                    hipLaunchKernelGGL(yfix_kernel, dim3((rows + 63) / 64), dim3(256), 0, s, n, j, i, rowpart, colpart, Vp,
                                       Wp, coef, y, seg);
                } else {
                    const int row_blocks = std::min(512, even ? ((rows + 1) / 2 + 3) / 4 : (rows + 3) / 4);
                    if (even)
                        hipLaunchKernelGGL((symv_kernel<true>), dim3(row_blocks + i), dim3(256), 0, s, A, n, j, row_blocks,
                                           vi, y, Vp, Wp, coef);
                    else
                        hipLaunchKernelGGL((symv_kernel<false>), dim3(row_blocks + i), dim3(256), 0, s, A, n, j, row_blocks,
                                           vi, y, Vp, Wp, coef);
                    if (i > 0)
                        hipLaunchKernelGGL(pfix_kernel, dim3((rows + 255) / 256), dim3(256), 0, s, n, j, i, Vp, Wp, coef, y);
                }
                hipLaunchKernelGGL(w_kernel, dim3(1), dim3(1024), 0, s, n, j, tau_d, vi, y, wi);
            }
            const int jn = j0 + nb;
            const int tiles = (n - jn + 63) / 64;
            hipLaunchKernelGGL(syr2k_kernel, dim3(tiles, tiles), dim3(256), 0, s, A, n, jn, nb, Vp, Wp, upper ? 1 : 0);
            LPD_HIP(hipGetLastError());
        }
        if (n >= 2) {
            hipLaunchKernelGGL(tri_tail_kernel, dim3(1), dim3(64), 0, s, A, n, dg_d, e_d);
        } else {
            LPD_HIP(hipMemcpyAsync(dg_d, A, 8, hipMemcpyDeviceToDevice, s));
        }
        LPD_HIP(hipGetLastError());
        LPD_HIP(hipMemcpyAsync(dge_h, dg_d, size_t(n) * 8, hipMemcpyDeviceToHost, s));
        LPD_HIP(hipMemcpyAsync(dge_h + n, e_d, size_t(n) * 8, hipMemcpyDeviceToHost, s));
        LPD_HIP(hipEventRecord(tri_done, s));
    }

    say("accumulation of the reflectors");
    // Q^T into Zt while the host starts on the tridiagonal matrix
    {
        double *Ypart = reinterpret_cast<double *>(ws + cv.off_Y);
        double *Y2 = Ypart + size_t(PA_KS) * size_t(n) * NB;
        hipLaunchKernelGGL(identity_kernel, dim3(2048), dim3(256), 0, s, Zt, n);
        const int nref = n - 2;
        const int npanel = nref > 0 ? (nref + NB - 1) / NB : 0;
        for (int pi = npanel - 1; pi >= 0; --pi) {
            const int k0 = pi * NB;
            const int nb = std::min(NB, nref - k0);
            const int nchunks = (n - (k0 + 1) + 127) / 128;
            hipLaunchKernelGGL(panel_gram_kernel, dim3(nchunks), dim3(256), 0, s, A, n, k0, nb, P);
            hipLaunchKernelGGL(panel_t_kernel, dim3(1), dim3(NB * NB), 0, s, P, nchunks, k0, nb, tau_d, T);
            // rows up to k0 are still unit vectors with nothing in the columns this panel touches
            const int r0 = k0 + 1;
            const int nrows = n - r0;
            const int nblk = (nrows + PA_RB - 1) / PA_RB;
            hipLaunchKernelGGL(panel_y_kernel, dim3(nblk, PA_KS), dim3(256), 0, s, Zt, n, A, k0, nb, r0, nrows, Ypart);
            hipLaunchKernelGGL(panel_y2_kernel, dim3((nrows * NB + 255) / 256), dim3(256), 0, s, Ypart, nrows, T, Y2);
            hipLaunchKernelGGL(panel_update_kernel, dim3(nblk, (nrows + 127) / 128), dim3(256), 0, s, Zt, n, A, k0, nb, r0,
                               nrows, Y2);
        }
        LPD_HIP(hipGetLastError());
    }

    LPD_HIP(hipEventSynchronize(tri_done));     // dg, e on the host; the panel kernels queued behind them keep running
    std::memcpy(dg.data(), dge_h, size_t(n) * 8);
    std::memcpy(e.data(), dge_h + n, size_t(n) * 8);
    if (n == 1) e[0] = 0.0;

    say("QL iteration (host) with rotation passes (device)");
    if (levels == 0) {
        ql[0].row0 = 0; ql[0].sz = n;
        ql[0].run(dg.data(), e.data());
        if (ql[0].hip_fail) { status = ql[0].hip_fail == 1 ? LPD_ERR_HIP : LPD_ERR_NUMERIC; goto done; }
        if (!ql[0].ok) { status = LPD_ERR_NUMERIC; goto done; }
    } else {
        // Tear the matrix into 2^levels leaves.  A tear at row m takes rho = |e_{m-1}| off the two diagonal entries
        // next to it and cuts the coupling; what it removed returns in its merge as rho u u^T with
        // u = e_{m-1} + sign e_m.  Q u = row (m - 1) + sign * row m of Q^T is saved now, before any rotation.
        {
            struct Span { int r0, sz, level; };
            std::vector<Span> stack{{0, n, levels}};
            std::vector<Tear> pre;                                    // parents before children
            while (!stack.empty()) {
                const Span sp = stack.back();
                stack.pop_back();
                if (sp.level == 0) { leaves.push_back({sp.r0, sp.sz}); continue; }
                const int m = sp.r0 + sp.sz / 2;
                Tear t{sp.r0, sp.sz, m, std::fabs(e[size_t(m) - 1]), e[size_t(m) - 1] < 0.0 ? -1.0 : 1.0, nullptr};
                pre.push_back(t);
                stack.push_back({m, sp.r0 + sp.sz - m, sp.level - 1});
                stack.push_back({sp.r0, m - sp.r0, sp.level - 1});
            }
            std::sort(leaves.begin(), leaves.end());
            tears.assign(pre.rbegin(), pre.rend());                   // every parent now comes after its children
        }
        for (size_t t = 0; t < tears.size(); ++t) {
            Tear &tr = tears[t];
            tr.uq = reinterpret_cast<double *>(ws + cv.off_uq + t * vec);
            dg[size_t(tr.m) - 1] -= tr.rho;
            dg[size_t(tr.m)] -= tr.rho;
            e[size_t(tr.m) - 1] = 0.0;
            hipLaunchKernelGGL(dc_save_u_kernel, dim3((n + 255) / 256), dim3(256), 0, s, Zt, n, tr.m, tr.sgn, tr.uq);
        }
        LPD_HIP(hipGetLastError());
        // one QL iteration per leaf, each on its own host thread and its own rows of dg, e and Zt
        {
            std::vector<std::thread> workers;
            for (int q = 0; q < nleaves; ++q) {
                ql[q].row0 = leaves[size_t(q)].first;
                ql[q].sz = leaves[size_t(q)].second;
            }
            for (int q = 1; q < nleaves; ++q)
                workers.emplace_back([&, q]() { ql[q].run(dg.data() + ql[q].row0, e.data() + ql[q].row0); });
            ql[0].run(dg.data() + ql[0].row0, e.data() + ql[0].row0);
            for (auto &w : workers) w.join();
        }
        for (int q = 0; q < nleaves; ++q) {
            if (ql[q].hip_fail) { status = ql[q].hip_fail == 1 ? LPD_ERR_HIP : LPD_ERR_NUMERIC; goto done; }
            if (!ql[q].ok) { status = LPD_ERR_NUMERIC; goto done; }
        }
        {
            auto dcv = [&](int k) { return ws + cv.off_dc + size_t(k) * vec; };
            DcBuffers bufs;
            bufs.Zt = Zt; bufs.U = A; bufs.G = reinterpret_cast<double *>(ws + cv.off_G);
            bufs.z = reinterpret_cast<double *>(dcv(1));
            bufs.dk = reinterpret_cast<double *>(dcv(2)); bufs.zk = reinterpret_cast<double *>(dcv(3));
            bufs.mu = reinterpret_cast<double *>(dcv(4)); bufs.zhat = reinterpret_cast<double *>(dcv(5));
            bufs.inv_norm = reinterpret_cast<double *>(dcv(6)); bufs.rotcs = reinterpret_cast<double *>(dcv(7));   // 2 n doubles
            bufs.org = reinterpret_cast<int *>(dcv(9)); bufs.rows = reinterpret_cast<int *>(dcv(10));
            bufs.ra = reinterpret_cast<int *>(dcv(11)); bufs.rb = reinterpret_cast<int *>(dcv(12));
            for (const Tear &tr : tears) {
                if (!(tr.rho > 0.0)) continue;              // the halves were never coupled
                status = dc_merge(n, tr, dg, bufs, g_staging.dc_h, s, talk);
                if (status != LPD_OK) goto done;
            }
        }
    }

    say("ordering and scaling");
    r = lpd_host::order_and_clip(dg.data(), n, clip_ratio, ord, eig_host);
    if (r < 0) { status = LPD_ERR_NUMERIC; goto done; }
    {
        // order (int32) and sorted eigenvalues through the page-locked block, after all rotation copies
        LPD_HIP(hipStreamSynchronize(s));
        int *ord_h = reinterpret_cast<int *>(dge_h);
        double *lam_h = dge_h + n;
        for (int j = 0; j < n; ++j) { ord_h[j] = int(ord[size_t(j)]); lam_h[j] = dg[size_t(ord[size_t(j)])]; }
        LPD_HIP(hipMemcpyAsync(ord_d, ord_h, size_t(n) * 4, hipMemcpyHostToDevice, s));
        LPD_HIP(hipMemcpyAsync(lam_d, lam_h, size_t(n) * 8, hipMemcpyHostToDevice, s));
        hipLaunchKernelGGL(finish_kernel, dim3(n), dim3(256), 0, s, Zt, n, ord_d, lam_d, int(r), W, ldw);
        LPD_HIP(hipGetLastError());
    }
    *rank = r;
    say("done");
done:
    if (hipStreamSynchronize(s) != hipSuccess && status == LPD_OK) status = LPD_ERR_HIP;
    return status;
}
