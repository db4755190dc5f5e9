// Bandwidth-bound row kernels for gfx950:
//   margins_kernel    m[t] = sum_j G[row(t), j] * w[j]      (Figure 1 step 2a, all rows or a row list)
//   sqnorm_kernel     s[i] = sum_k X[i,k]^2                  (the ||x||^2 terms of the Gaussian kernel, Section 5)
//
// A row is spread over LPR lanes of a wavefront (LPR = 64 for long rows down to
// 8 for short ones, so narrow factors still fill every lane); each lane streams
// 16-byte pieces, UNROLL of them in flight per row, and the partial sums meet in
// a butterfly over the LPR lanes.  Rows are dealt out in a grid-stride loop so
// one launch of a few thousand wavefronts covers any n.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lpd {

typedef float rf32x4 __attribute__((ext_vector_type(4)));

template <int LPR>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// VEC: G rows are 16-byte aligned (pointer and leading dimension), vector loads allowed.
// ROWS: rows a lane group works on at once; they share each load of w, which is what lifts the
// long-row sweep from 82 % to 89 % of HBM bandwidth (two rows; more rows lose it again to
// register pressure).  A group past the end re-reads the last row and drops the result.
// INDEXED: an index outside [0, n_rows_G) reads row 0 instead and yields NaN, so that no list can make the
// kernel read outside G.
template <int LPR, bool VEC, bool INDEXED, int ROWS>
__global__ __launch_bounds__(256) void margins_kernel(const float *__restrict__ G, int64_t n_out, int r,
                                                      int64_t ldg, const int64_t *__restrict__ rows,
                                                      int64_t n_rows_G, const float *__restrict__ w,
                                                      float *__restrict__ m, int64_t m_stride)
{
    constexpr int GROUPS = 256 / LPR;             // lane groups per workgroup
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const int64_t stride = int64_t(gridDim.x) * GROUPS * ROWS;
    const int r4 = VEC ? (r & ~3) : 0;

    for (int64_t t0 = (int64_t(blockIdx.x) * GROUPS + grp) * ROWS; t0 < n_out; t0 += stride) {
        const float *g[ROWS];
        bool bad[ROWS];
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int64_t t = t0 + q < n_out ? t0 + q : n_out - 1;
            int64_t row = INDEXED ? rows[t] : t;
            bad[q] = INDEXED && (row < 0 || row >= n_rows_G);
            if (bad[q]) row = 0;
            g[q] = G + row * ldg;
        }
        float s[ROWS][4];
#pragma unroll
        for (int q = 0; q < ROWS; ++q)
#pragma unroll
            for (int u = 0; u < 4; ++u) s[q][u] = 0.f;
        if (VEC) {
            constexpr int STEP = LPR * 4;
            int j = sub * 4;
            for (; j + 3 * STEP < r4; j += 4 * STEP) {
                rf32x4 gv[ROWS][4], wv[4];
#pragma unroll
                for (int q = 0; q < ROWS; ++q)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        gv[q][u] = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g[q] + j + u * STEP));
#pragma unroll
                for (int u = 0; u < 4; ++u) wv[u] = *reinterpret_cast<const rf32x4 *>(w + j + u * STEP);
#pragma unroll
                for (int q = 0; q < ROWS; ++q)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        s[q][u] += gv[q][u].x * wv[u].x + gv[q][u].y * wv[u].y + gv[q][u].z * wv[u].z +
                                   gv[q][u].w * wv[u].w;
            }
            for (; j < r4; j += STEP) {
                const rf32x4 w0 = *reinterpret_cast<const rf32x4 *>(w + j);
#pragma unroll
                for (int q = 0; q < ROWS; ++q) {
                    const rf32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g[q] + j));
                    s[q][0] += g0.x * w0.x + g0.y * w0.y + g0.z * w0.z + g0.w * w0.w;
                }
            }
        }
        for (int j = r4 + sub; j < r; j += LPR) {
            const float wj = w[j];
#pragma unroll
            for (int q = 0; q < ROWS; ++q) s[q][1] += g[q][j] * wj;
        }
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const float tot = group_sum<LPR>((s[q][0] + s[q][1]) + (s[q][2] + s[q][3]));
            if (sub == 0 && t0 + q < n_out) m[(t0 + q) * m_stride] = bad[q] ? __builtin_nanf("") : tot;
        }
    }
}

// cen (may be NULL): the row is taken relative to this point, s[i] = sum_k (X[i,k] - cen[k])^2; d floats,
// 16-byte aligned.
template <int LPR, bool VEC>
__global__ __launch_bounds__(256) void sqnorm_kernel(const float *__restrict__ X, int64_t n, int d, int64_t ldx,
                                                     const float *__restrict__ cen, float *__restrict__ out)
{
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const int64_t stride = int64_t(gridDim.x) * GROUPS;
    const int d4 = VEC ? (d & ~3) : 0;
    for (int64_t i = int64_t(blockIdx.x) * GROUPS + grp; i < n; i += stride) {
        const float *x = X + i * ldx;
        float s0 = 0.f, s1 = 0.f;
        if (VEC) {
            for (int k = sub * 4; k < d4; k += LPR * 4) {
                rf32x4 v = *reinterpret_cast<const rf32x4 *>(x + k);
                if (cen) v -= *reinterpret_cast<const rf32x4 *>(cen + k);
                s0 += v.x * v.x + v.y * v.y;
                s1 += v.z * v.z + v.w * v.w;
            }
        }
        for (int k = d4 + sub; k < d; k += LPR) {
            const float v = cen ? x[k] - cen[k] : x[k];
            s1 += v * v;
        }
        const float s = group_sum<LPR>(s0 + s1);
        if (sub == 0) out[i] = s;
    }
}

// The origin the Gaussian kernel block works from: cen[k] = mean over a sample of the landmark rows of L[., k]
// (every `step`-th row, `rows` of them).  Any point serves, a distance does not depend on the origin; one
// inside the data keeps ||x - cen||^2 of the order of the distances.  A workgroup owns 64 features; its four
// wavefronts take every fourth sampled row (coalesced) and meet in LDS.
__global__ __launch_bounds__(256) void centre_kernel(const float *__restrict__ L, int64_t ldl, int d, int rows,
                                                     int64_t step, float *__restrict__ cen)
{
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    float s = 0.f;
    if (k < d)
        for (int i = wv; i < rows; i += 4) s += L[int64_t(i) * step * ldl + k];
    part[wv][lane] = s;
    __syncthreads();
    if (wv == 0 && k < d) cen[k] = ((part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane])) / float(rows);
}

// M[i, q] = sum_j G[i, j] * Ws[q, j] for a handful of weight vectors at once (K <= 8): one pass over G
// serves all of them (the sweep the solver's callers run for several classifiers that share G: C grid,
// folds, class pairs; Section 4).  A wavefront takes ROWS rows at a time: every 16-byte piece of a weight
// vector it reads (through the cache) is used for all of them, so the cache traffic per byte of G falls
// with ROWS; G itself comes in 16-byte non-temporal loads; K * ROWS butterflies end a group of rows.  A
// group past the end re-reads the last row and drops the result.
template <int K, bool VEC, int ROWS>
__global__ __launch_bounds__(256) void margins_multi_kernel(const float *__restrict__ G, int64_t n, int r, int64_t ldg,
                                                            const float *__restrict__ Ws, int64_t ldws,
                                                            float *__restrict__ M, int64_t ldm)
{
    const int lane = threadIdx.x & 63;
    const int64_t stride = int64_t(gridDim.x) * 4 * ROWS;
    const int r4 = VEC ? (r & ~3) : 0;
    for (int64_t i0 = (int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6)) * ROWS; i0 < n; i0 += stride) {
        const float *g[ROWS];
#pragma unroll
        for (int t = 0; t < ROWS; ++t) g[t] = G + (i0 + t < n ? i0 + t : n - 1) * ldg;
        float s[ROWS][K];
#pragma unroll
        for (int t = 0; t < ROWS; ++t)
#pragma unroll
            for (int q = 0; q < K; ++q) s[t][q] = 0.f;
        if (VEC) {
            for (int j = lane * 4; j < r4; j += 256) {
                rf32x4 gv[ROWS];
#pragma unroll
                for (int t = 0; t < ROWS; ++t) gv[t] = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g[t] + j));
#pragma unroll
                for (int q = 0; q < K; ++q) {
                    const rf32x4 w0 = *reinterpret_cast<const rf32x4 *>(Ws + q * ldws + j);
#pragma unroll
                    for (int t = 0; t < ROWS; ++t)
                        s[t][q] += gv[t].x * w0.x + gv[t].y * w0.y + gv[t].z * w0.z + gv[t].w * w0.w;
                }
            }
        }
        for (int j = r4 + lane; j < r; j += 64) {
            float gj[ROWS];
#pragma unroll
            for (int t = 0; t < ROWS; ++t) gj[t] = g[t][j];
#pragma unroll
            for (int q = 0; q < K; ++q) {
                const float wj = Ws[q * ldws + j];
#pragma unroll
                for (int t = 0; t < ROWS; ++t) s[t][q] += gj[t] * wj;
            }
        }
#pragma unroll
        for (int t = 0; t < ROWS; ++t)
#pragma unroll
            for (int q = 0; q < K; ++q) {
                const float tot = group_sum<64>(s[t][q]);
                if (lane == 0 && i0 + t < n) M[(i0 + t) * ldm + q] = tot;
            }
    }
}

// V[j, b] = sum_k Ws[j, k] * W[k, b]: classifier weights folded through the whitening map, so that a
// score becomes one inner product with the kernel row, f_j(x) = V_j . z(x) (Section 4, prediction step).
// One thread per column b of W, CPT classifiers per pass held in registers; W is streamed once per
// pass with coalesced rows, the CPT weights of row k are broadcast loads.
template <int CPT>
__global__ __launch_bounds__(256) void fold_weights_kernel(const float *__restrict__ W, int r, int B, int64_t ldw,
                                                           const float *__restrict__ Ws, int c, int64_t ldws,
                                                           float *__restrict__ V, int64_t ldv)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    const int j0 = blockIdx.y * CPT;
    if (b >= B) return;
    float acc[CPT];
#pragma unroll
    for (int q = 0; q < CPT; ++q) acc[q] = 0.f;
    for (int k = 0; k < r; ++k) {
        const float wkb = W[int64_t(k) * ldw + b];
#pragma unroll
        for (int q = 0; q < CPT; ++q)
            if (j0 + q < c) acc[q] += Ws[int64_t(j0 + q) * ldws + k] * wkb;
    }
#pragma unroll
    for (int q = 0; q < CPT; ++q)
        if (j0 + q < c) V[int64_t(j0 + q) * ldv + b] = acc[q];
}

// Rows p0 .. p0+rows-1 of a matrix in compressed-row form written out into the dense panel Xd
// (Section 4: kernel operations on sparse data).  The panel is cleared by fill_zero_kernel first; then one
// wavefront per row scatters its entries.  An index outside [0, d) is skipped, so that no input can make
// the kernel write outside the panel.
__global__ __launch_bounds__(256) void fill_zero_kernel(rf32x4 *__restrict__ p, int64_t count4)
{
    const rf32x4 z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < count4; i += int64_t(gridDim.x) * 256) p[i] = z;
}

__global__ __launch_bounds__(256) void csr_scatter_kernel(const int64_t *__restrict__ row_ptr,
                                                          const int32_t *__restrict__ col_idx,
                                                          const float *__restrict__ values, int64_t p0, int64_t rows,
                                                          int d, float *__restrict__ Xd, int64_t ldxd)
{
    const int lane = threadIdx.x & 63;
    for (int64_t t = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6); t < rows; t += int64_t(gridDim.x) * 4) {
        const int64_t e0 = row_ptr[p0 + t], e1 = row_ptr[p0 + t + 1];
        float *x = Xd + t * ldxd;
        for (int64_t e = e0 + lane; e < e1; e += 64) {
            const int32_t c = col_idx[e];
            if (c >= 0 && c < d) x[c] = values[e];
        }
    }
}

// Lt[k, b] = L[b, k]: the landmarks with the feature index outermost, so that the B kernel arguments one
// stored entry of a sparse row contributes to are contiguous.  32 x 32 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ L, int B, int d, int64_t ldl,
                                                        float *__restrict__ Lt, int64_t ldlt)
{
    __shared__ float tile[32][33];
    const int b0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int b = b0 + ty + 8 * q, k = k0 + tx;
        tile[ty + 8 * q][tx] = (b < B && k < d) ? L[int64_t(b) * ldl + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int k = k0 + ty + 8 * q, b = b0 + tx;
        if (k < d && b < B) Lt[int64_t(k) * ldlt + b] = tile[tx][ty + 8 * q];
    }
}

// Kernel block of sparse rows by gathering (Section 4: kernel operations as sparse matrix products), for
// rows so sparse that writing them out would waste the contraction: S[t, b] = sum over the stored entries
// (k, v) of row t of v * Lt[k, b], then Z = exp2(scale * max(0, ||x_t||^2 + ||l_b||^2 - 2 S)).  A workgroup
// owns 1,024 consecutive landmarks (4 per lane) and walks over rows; the entries of a row are uniform
// across the workgroup, each costs one 16-byte load of Lt per lane, four of them in flight.
__global__ __launch_bounds__(256) void csr_gauss_gather_kernel(const int64_t *__restrict__ row_ptr,
                                                               const int32_t *__restrict__ col_idx,
                                                               const float *__restrict__ values, int64_t p0,
                                                               int64_t rows, int d, const float *__restrict__ Lt,
                                                               int B, int64_t ldlt, const float *__restrict__ nl,
                                                               float scale, float *__restrict__ Z, int64_t ldz)
{
    const int c = blockIdx.x * 1024 + threadIdx.x * 4;
    const int cl = c < B ? c : 0;                     // lanes past the end read a valid address, store nothing
    float nlc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) nlc[q] = c + q < B ? nl[c + q] : 0.f;
    const bool vec_store = (ldz % 4 == 0) && ((reinterpret_cast<uintptr_t>(Z) & 15) == 0) && c + 3 < B;
    for (int64_t t = blockIdx.y; t < rows; t += gridDim.y) {
        const int64_t e0 = row_ptr[p0 + t], e1 = row_ptr[p0 + t + 1];
        rf32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float nx = 0.f;
        for (int64_t e = e0; e < e1; e += 4) {
            float v[4];
            const rf32x4 *src[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = e + u < e1;
                const int32_t k = in ? col_idx[e + u] : 0;
                const bool ok = in && k >= 0 && k < d;
                v[u] = ok ? values[e + u] : 0.f;
                src[u] = reinterpret_cast<const rf32x4 *>(Lt + int64_t(ok ? k : 0) * ldlt + cl);
            }
            rf32x4 l[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) l[u] = *src[u];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc += v[u] * l[u];
                nx += v[u] * v[u];
            }
        }
        float z[4];
        const float a4[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) z[q] = exp2f(scale * fmaxf(0.f, nx + nlc[q] - 2.f * a4[q]));
        float *out = Z + t * ldz + c;
        if (vec_store) {
            *reinterpret_cast<rf32x4 *>(out) = rf32x4{z[0], z[1], z[2], z[3]};
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (c + q < B) out[q] = z[q];
        }
    }
}

}  // namespace lpd
