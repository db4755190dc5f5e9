// Bandwidth-bound row kernels for gfx950:
//   margins_kernel    m[t] = sum_j G[row(t), j] * w[j]      (Figure 1 step 2a, all rows or a row list)
//   sqnorm_kernel     s[i] = sum_k X[i,k]^2                  (the ||x||^2 terms of the Gaussian kernel, Section 4)
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
template <int LPR, bool VEC, bool INDEXED>
__global__ __launch_bounds__(256) void margins_kernel(const float *__restrict__ G, int64_t n_out, int r,
                                                      int64_t ldg, const int64_t *__restrict__ rows,
                                                      const float *__restrict__ w, float *__restrict__ m)
{
    constexpr int GROUPS = 256 / LPR;             // rows in flight per workgroup
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const int64_t stride = int64_t(gridDim.x) * GROUPS;
    const int r4 = VEC ? (r & ~3) : 0;

    for (int64_t t = int64_t(blockIdx.x) * GROUPS + grp; t < n_out; t += stride) {
        const int64_t row = INDEXED ? rows[t] : t;
        const float *g = G + row * ldg;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        if (VEC) {
            constexpr int STEP = LPR * 4;
            int j = sub * 4;
            for (; j + 3 * STEP < r4; j += 4 * STEP) {
                const rf32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g + j));
                const rf32x4 g1 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g + j + STEP));
                const rf32x4 g2 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g + j + 2 * STEP));
                const rf32x4 g3 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g + j + 3 * STEP));
                const rf32x4 w0 = *reinterpret_cast<const rf32x4 *>(w + j);
                const rf32x4 w1 = *reinterpret_cast<const rf32x4 *>(w + j + STEP);
                const rf32x4 w2 = *reinterpret_cast<const rf32x4 *>(w + j + 2 * STEP);
                const rf32x4 w3 = *reinterpret_cast<const rf32x4 *>(w + j + 3 * STEP);
                s0 += g0.x * w0.x + g0.y * w0.y + g0.z * w0.z + g0.w * w0.w;
                s1 += g1.x * w1.x + g1.y * w1.y + g1.z * w1.z + g1.w * w1.w;
                s2 += g2.x * w2.x + g2.y * w2.y + g2.z * w2.z + g2.w * w2.w;
                s3 += g3.x * w3.x + g3.y * w3.y + g3.z * w3.z + g3.w * w3.w;
            }
            for (; j < r4; j += STEP) {
                const rf32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const rf32x4 *>(g + j));
                const rf32x4 w0 = *reinterpret_cast<const rf32x4 *>(w + j);
                s0 += g0.x * w0.x + g0.y * w0.y + g0.z * w0.z + g0.w * w0.w;
            }
        }
        for (int j = r4 + sub; j < r; j += LPR) s1 += g[j] * w[j];
        const float s = group_sum<LPR>((s0 + s1) + (s2 + s3));
        if (sub == 0) m[t] = s;
    }
}

template <int LPR, bool VEC>
__global__ __launch_bounds__(256) void sqnorm_kernel(const float *__restrict__ X, int64_t n, int d, int64_t ldx,
                                                     float *__restrict__ out)
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
                const rf32x4 v = *reinterpret_cast<const rf32x4 *>(x + k);
                s0 += v.x * v.x + v.y * v.y;
                s1 += v.z * v.z + v.w * v.w;
            }
        }
        for (int k = d4 + sub; k < d; k += LPR) s1 += x[k] * x[k];
        const float s = group_sum<LPR>(s0 + s1);
        if (sub == 0) out[i] = s;
    }
}

}  // namespace lpd
