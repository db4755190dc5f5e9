// Figure 1 step 1d in ONE launch for few landmarks (B <= 256): a workgroup takes 32 points, forms their
// row of the kernel block Z = exp(-gamma ||x - l||^2) (Section 5 kernel) in LDS and multiplies it by W^T
// right there, so Z never reaches memory and the four launches of the panel schedule (origin, two norm
// kernels, kernel block, whitening product) become one.  With so few landmarks those launches are
// latency-bound, and so is this one: the point is the launch count, not the inner loop, which is kept plain
// (one barrier pair per 16-wide slice, the next slice requested before the MFMAs of the current one).
//
//   phase 0  origin c = mean of up to 32 landmark rows spread evenly over L (any origin serves, a distance
//            does not depend on it; see the accuracy note in lpd.h), into LDS
//   phase 1  S = (X_strip - c)(L - c)^T over the d features with v_mfma_f32_32x32x2_f32, slices of 16
//            features staged through LDS; the squared norms of the shifted rows are summed from the very
//            registers that carry the slices
//   phase 2  Z = exp2(scale * max(0, ||x-c||^2 + ||l-c||^2 - 2 S)) from the accumulators into LDS, zero
//            beyond column B
//   phase 3  G_strip = Z W^T over the B landmarks, W in slices of 16 through the same LDS buffer
//   phase 4  G rows out, zero-filled from column r to B-1
//
// Operand layout of the MFMA as in gemm_nt.hip.h: lane l feeds row l%32 of both operands; lanes 0-31 carry
// k0..k0+3 and lanes 32-63 k0+4..k0+7 of an 8-wide step (one ds_read_b128 each); accumulator register v of
// lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lpd {

typedef float sf32x4 __attribute__((ext_vector_type(4)));
typedef float sf32x16 __attribute__((ext_vector_type(16)));

constexpr int SM_TM = 32;          // points per workgroup
constexpr int SM_MAXB = 256;       // landmarks (and outputs) this kernel handles
constexpr int SM_MAXD = 1024;      // features: the origin lives in LDS (61.6 KB of static LDS in all)
constexpr int SM_LDK = 16 + 4;     // floats per staged slice row
constexpr int SM_ZLD = SM_MAXB + 4;

struct SmallArgs {
    const float *X, *L, *W;
    float *G;
    int64_t ldx, ldl, ldw, ldg;
    int n, d, B, r;
    int cen_rows;       // landmark rows averaged for the origin
    int cen_step;       // spacing of those rows
    float scale;        // -gamma * log2(e)
};

// VEC: 16-byte loads allowed (X, L, W 16-byte aligned, leading dimensions, d and B multiples of 4)
template <bool VEC>
__global__ __launch_bounds__(256) void nystrom_small_kernel(SmallArgs p)
{
    __shared__ __attribute__((aligned(16))) float Ls[SM_MAXB * SM_LDK];   // a slice of L, later of W
    __shared__ __attribute__((aligned(16))) float Xs[SM_TM * SM_LDK];
    __shared__ __attribute__((aligned(16))) float Zs[SM_TM * SM_ZLD];
    __shared__ __attribute__((aligned(16))) float cen[SM_MAXD];
    __shared__ float nxs[SM_TM], nls[SM_MAXB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.x * SM_TM;
    const int lrow = tid >> 2, lch = tid & 3;       // loader: row within a pass of 64 rows, 4-float chunk

    // ---- phase 0: origin
    for (int k = tid; k < p.d; k += 256) {
        float s = 0.f;
        for (int i = 0; i < p.cen_rows; ++i) s += p.L[int64_t(i) * p.cen_step * p.ldl + k];
        cen[k] = s / float(p.cen_rows);
    }
    __syncthreads();

    // one 4-float chunk of a row, shifted by the origin, zero beyond column `lim`
    auto load4 = [&](const float *row, int k, int lim, bool shift) __attribute__((always_inline)) -> sf32x4 {
        sf32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (VEC) {
            if (k < lim) {
                v = *reinterpret_cast<const sf32x4 *>(row + k);
                if (shift) v -= *reinterpret_cast<const sf32x4 *>(&cen[k]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < lim) v[e] = shift ? row[k + e] - cen[k + e] : row[k + e];
        }
        return v;
    };

    // ---- phase 1: S = (X - c)(L - c)^T, wave w owns landmark tiles w and w + 4
    const float *xrow = p.X + int64_t(min(m0 + lrow, p.n - 1)) * p.ldx;       // threads 0..127 load X
    const float *lrowp[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) lrowp[q] = p.L + int64_t(min(lrow + 64 * q, p.B - 1)) * p.ldl;
    sf32x16 acc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
    float sx = 0.f, sl[4] = {0.f, 0.f, 0.f, 0.f};
    const int frag = (lane & 31) * SM_LDK + (lane >> 5) * 4;
    // the next slice is requested before the MFMAs of the current one, so its trip to memory overlaps them
    sf32x4 xv = {0.f, 0.f, 0.f, 0.f}, lv[4];
    auto fetch1 = [&](int k0) __attribute__((always_inline)) {
        const int k = k0 + lch * 4;
        if (tid < 128) xv = load4(xrow, k, p.d, true);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (64 * q < p.B) lv[q] = load4(lrowp[q], k, p.d, true);
    };
    if (p.d > 0) fetch1(0);
    for (int k0 = 0; k0 < p.d; k0 += 16) {
        if (tid < 128) {
            sx += (xv.x * xv.x + xv.y * xv.y) + (xv.z * xv.z + xv.w * xv.w);
            *reinterpret_cast<sf32x4 *>(&Xs[lrow * SM_LDK + lch * 4]) = xv;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (64 * q < p.B) {
                const sf32x4 v = lv[q];
                sl[q] += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
                *reinterpret_cast<sf32x4 *>(&Ls[(lrow + 64 * q) * SM_LDK + lch * 4]) = v;
            }
        }
        __syncthreads();
        if (k0 + 16 < p.d) fetch1(k0 + 16);
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const sf32x4 a = *reinterpret_cast<const sf32x4 *>(&Xs[frag + kc * 8]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int jt = wave + 4 * u;
                if (jt * 32 < p.B) {
                    const sf32x4 b = *reinterpret_cast<const sf32x4 *>(&Ls[jt * 32 * SM_LDK + frag + kc * 8]);
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc[u], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }
    // norms: the four chunk owners of a row sit in adjacent lanes
    sx += __shfl_xor(sx, 1, 64);
    sx += __shfl_xor(sx, 2, 64);
    if (tid < 128 && lch == 0) nxs[lrow] = sx;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float s = sl[q];
        s += __shfl_xor(s, 1, 64);
        s += __shfl_xor(s, 2, 64);
        if (lch == 0) nls[lrow + 64 * q] = s;
    }
    __syncthreads();

    // ---- phase 2: Z into LDS, zero beyond column B (the contraction below runs to the next multiple of 16)
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int jt = wave + 4 * u;
        if (jt * 32 < p.B) {
            const int col = jt * 32 + col_in;
            const float nb = nls[col];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 8 * (v >> 2) + row_in + (v & 3);
                const float dist = fmaxf(nxs[row] + nb - 2.0f * acc[u][v], 0.0f);
                Zs[row * SM_ZLD + col] = col < p.B ? __builtin_amdgcn_exp2f(p.scale * dist) : 0.0f;
            }
        }
    }
    __syncthreads();

    // ---- phase 3: G = Z W^T, wave w owns output tiles w and w + 4
    const float *wrowp[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) wrowp[q] = p.W + int64_t(min(lrow + 64 * q, max(p.r - 1, 0))) * p.ldw;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
    auto fetch3 = [&](int k0) __attribute__((always_inline)) {
        const int k = k0 + lch * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (64 * q < p.r) lv[q] = load4(wrowp[q], k, p.B, false);
    };
    if (p.r > 0) fetch3(0);
    for (int k0 = 0; k0 < p.B && p.r > 0; k0 += 16) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (64 * q < p.r) *reinterpret_cast<sf32x4 *>(&Ls[(lrow + 64 * q) * SM_LDK + lch * 4]) = lv[q];
        __syncthreads();
        if (k0 + 16 < p.B) fetch3(k0 + 16);
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const sf32x4 a = *reinterpret_cast<const sf32x4 *>(&Zs[(lane & 31) * SM_ZLD + k0 + kc * 8 + (lane >> 5) * 4]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int jt = wave + 4 * u;
                if (jt * 32 < p.r) {
                    const sf32x4 b = *reinterpret_cast<const sf32x4 *>(&Ls[jt * 32 * SM_LDK + frag + kc * 8]);
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc[u], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    // ---- phase 4: rows of G; columns r..B-1 are zeros
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int jt = wave + 4 * u;
        if (jt * 32 >= p.B) continue;
        const int col = jt * 32 + col_in;
        if (col >= p.B) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + 8 * (v >> 2) + row_in + (v & 3);
            if (row < p.n) p.G[int64_t(row) * p.ldg + col] = col < p.r ? acc[u][v] : 0.0f;
        }
    }
}

}  // namespace lpd
