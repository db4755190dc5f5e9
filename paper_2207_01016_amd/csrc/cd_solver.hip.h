// Dual coordinate ascent with shrinking on the rows of the factor G, many
// independent binary problems at once (Section 2, equation (2) and the truncated
// Newton step; Section 4, "Shrinking"; Figure 1 steps 2a-2b).
//
//   maximise  sum_i alpha_i - 1/2 ||w||^2,  0 <= alpha_i <= C,  w = sum_i alpha_i y_i g_i
//   step on i:  f = g_i . w (2a);  alpha_i <- clip(alpha_i + (1 - y_i f) / ||g_i||^2, 0, C);
//               w <- w + (alpha_new - alpha_old) y_i g_i (2b)
//
// The loop is sequential inside a problem (the paper keeps one problem on one
// multiprocessor with w in its scratchpad); the parallelism is across problems
// (grid search, folds, one-versus-one pairs share one G).  Mapping for CDNA4:
//   * one problem = one workgroup of WAVES wavefronts (1 for r <= 4096, 4 above);
//     w and the current row of G live in registers, 4*NCH consecutive-by-lane
//     columns per lane, so the row load is one coalesced 16-byte access per lane
//     and chunk, the inner product ends in a butterfly over the 64 lanes (plus a
//     4-entry LDS exchange when WAVES = 4), and the update of w reuses the row
//     registers: G is read once per step, 4r bytes.
//   * everything that depends only on the visiting order -- variable index, row
//     index, label, alpha, unchanged-counter, ||g||^2 -- is gathered for 64 steps
//     at a time, one step per lane, into LDS; the next row of G is requested
//     before the current step's reduction.  Only the reduction and a handful of
//     scalar operations sit on the dependent path of a step.
//   * every lane executes the scalar logic on identical values (the butterfly
//     leaves the same bits in all lanes), so control flow is uniform; one lane
//     writes alpha, counters and the lists.
//
// Shrinking and stopping rule (Section 4, "Shrinking", fixes k = 5 and eta = 5 %;
// the stopping criterion is named there as a standard one and not spelled out).
// The reading implemented here:
//   - round-robin over the active list (initially the caller's order), one pass
//     = one epoch; a variable whose step left alpha bit-for-bit unchanged k times
//     in a row moves to a FIFO queue of removed variables;
//   - after every S = round((1-eta)/eta) active steps one step goes to the head of
//     that queue: if it changes alpha the variable rejoins the next epoch's list,
//     else it returns to the tail;
//   - violation before a step: max(grad,0) at alpha = 0, max(-grad,0) at alpha = C,
//     |grad| inside; when an epoch's largest violation is <= eps, w is recomputed
//     from alpha (the incremental updates drift in fp32), all removed variables
//     are swept with that w, violators rejoin; the problem is solved when there
//     are none and the epoch itself had started from a recomputed w.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lpd {

typedef float cf32x4 __attribute__((ext_vector_type(4)));

struct CdStatus {          // one per problem, mirrors lpd_cd_status
    int64_t steps;         // inner products spent (active steps + re-checks + final sweeps)
    int32_t epochs;
    int32_t converged;
    int32_t active;        // size of the active list at exit
    float max_violation;   // largest violation seen in the last epoch
    float dual;            // sum alpha - 1/2 ||w||^2
    int32_t reserved;
};

struct CdArgs {
    const float *G; int64_t ldg; int r;
    int64_t n;                      // rows of G: listed row indices are clamped to [0, n)
    const float *gsq;               // ||g_i||^2 per row of G
    const int64_t *prob_off;        // n_problems + 1 offsets into rows / y / alpha
    const int64_t *rows;            // concatenated row lists (visiting order)
    const float *y;                 // +-1 per listed row
    const float *C;                 // per problem
    float *alpha;                   // in: start (warm start), out: solution
    float *w; int64_t ldw;          // n_problems x r out
    CdStatus *status;
    int32_t *lists;                 // 3 * (total + n_problems) ints: active, next, removed
    uint8_t *cnt;                   // total bytes: unchanged-counters
    int64_t total;                  // prob_off[n_problems]
    int64_t n_problems;
    float eps; int max_epochs; int shrink_k; int check_every;   // check_every = S, 0 = no re-checks
};

// The lists, alpha and the counters are written by one lane and read back later by other lanes of
// the same workgroup only: workgroup-scope atomics and fences are enough (one CU, one vector L1),
// and unlike device-scope ones they cost no L2 write-back or invalidate.
template <typename T>
__device__ __forceinline__ T ld_wg(const T *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
template <typename T>
__device__ __forceinline__ void st_wg(T *p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ void wg_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __syncthreads();
}

// Sum over the 64 lanes, returned as one wave-uniform value.  Data-parallel-primitive moves inside
// the VALU (no LDS round trips): two quad permutes, half-row and row mirrors leave each row of 16
// lanes holding its total; row broadcasts carry lane 15 into the next row and lane 31 into the upper
// two rows, so lane 63 ends with the full sum, which is read into a scalar register.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false);
    return v + __builtin_bit_cast(float, moved);
}
__device__ __forceinline__ float wave_allsum(float v)
{
    v = dpp_add<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141, 0xf>(v);   // row_half_mirror
    v = dpp_add<0x140, 0xf>(v);   // row_mirror
    v = dpp_add<0x142, 0xa>(v);   // row_bcast15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);   // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ float cd_violation(float alpha, float grad, float C)
{
    if (alpha <= 0.0f) return fmaxf(grad, 0.0f);
    if (alpha >= C) return fmaxf(-grad, 0.0f);
    return fabsf(grad);
}

// VEC: rows of G are 16-byte aligned (pointer and leading dimension); otherwise element-wise loads.
// MODE 0: rows read element-wise (any alignment); 1: 16-byte row loads; 2: 16-byte loads and r equal to the
// 4 * NCH * 64 * WAVES columns the lanes cover, so that no lane ever holds a column past the end.
template <int WAVES, int NCH, int MODE>
__global__ __launch_bounds__(64 * WAVES) void cd_solve_kernel(CdArgs a)
{
    constexpr bool VEC = MODE != 0;
    constexpr bool EXACT = MODE == 2;
    constexpr int T = 64 * WAVES;
    constexpr int BLK = 64;                  // steps whose metadata is gathered at once
    // row buffers in flight.  Measured on 1,125 problems of rank 1,024: 2 -> 165 ms, 4 -> 148, 6 -> 143, 8 -> 185
    // (the step loop is unrolled D times for static register indexing; past 6 the code and the registers
    // it needs cost more than the deeper prefetch gains)
    constexpr int D = NCH <= 4 ? 6 : NCH <= 8 ? 4 : 2;
    __shared__ int32_t s_t[BLK];
    __shared__ int64_t s_row[BLK];
    __shared__ float s_y[BLK], s_alpha[BLK], s_q[BLK];
    __shared__ int32_t s_cnt[BLK];
    __shared__ float s_part[2][WAVES];

    const int p = blockIdx.x;
    const int gl = threadIdx.x;
    const int wave = gl >> 6;
    // offsets and row indices come from the caller's device memory unchecked by the host: they are clamped
    // here, so that no content of those arrays can take an access outside the lists or outside G (a problem
    // with clamped entries solves something other than what the caller meant; its memory accesses stay legal)
    const int64_t o0 = min(max(a.prob_off[p], int64_t(0)), a.total);
    const int np = int(min(max(a.prob_off[p + 1] - o0, int64_t(0)), a.total - o0));
    const int64_t *rows = a.rows + o0;
    const int64_t row_max = a.n - 1;
    auto row_of = [&](int t) __attribute__((always_inline)) -> int64_t { return min(max(rows[t], int64_t(0)), row_max); };
    const float *y = a.y + o0;
    float *alpha = a.alpha + o0;
    uint8_t *cnt = a.cnt + o0;
    const int64_t stride = a.total + a.n_problems;
    // the three lists of this problem as offsets from one base pointer (the roles of the first two
    // swap after every epoch; swapping integers keeps all list accesses plain global accesses)
    int32_t *const lb = a.lists + (o0 + p);
    int64_t o_act = 0, o_nxt = stride;      // recomputed from the epoch parity, never swapped
    const int64_t o_rem = 2 * stride;
    const int cap = np + 1;
    const float C = a.C[p];
    const int r = a.r;

    // lane -> columns: chunk c covers columns (c*T + gl)*4 .. +3.  Loads are bare loads: nothing
    // touches a loaded register before the step that consumes it, so they stay in flight.  Chunks
    // (or chunk tails) past column r are read from a valid address and zeroed when consumed.
    int nvalid[NCH], coff[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * T + gl) * 4;
        nvalid[c] = min(max(r - col, 0), 4);
        coff[c] = nvalid[c] > 0 ? col : 0;
    }
    auto load_row = [&](cf32x4(&g)[NCH], int64_t row) __attribute__((always_inline)) {
        const float *base = a.G + row * a.ldg;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (VEC) {
                g[c] = *reinterpret_cast<const cf32x4 *>(base + coff[c]);
            } else {
                const float *e = base + coff[c];
                g[c].x = e[0];
                g[c].y = e[nvalid[c] > 1 ? 1 : 0];
                g[c].z = e[nvalid[c] > 2 ? 2 : 0];
                g[c].w = e[nvalid[c] > 3 ? 3 : 0];
            }
        }
    };
    auto valid = [&](const cf32x4(&g)[NCH], int c) __attribute__((always_inline)) -> cf32x4 {
        cf32x4 v = g[c];
        if (!EXACT) {
            if (nvalid[c] < 1) v.x = 0.f;
            if (nvalid[c] < 2) v.y = 0.f;
            if (nvalid[c] < 3) v.z = 0.f;
            if (nvalid[c] < 4) v.w = 0.f;
        }
        return v;
    };
    int parity = 0;
    auto block_sum = [&](float part) __attribute__((always_inline)) -> float {
        float s = wave_allsum(part);
        if (WAVES > 1) {
            if ((gl & 63) == 0) s_part[parity][wave] = s;
            __syncthreads();
            s = 0.f;
#pragma unroll
            for (int v = 0; v < WAVES; ++v) s += s_part[parity][v];
            parity ^= 1;
        }
        return s;
    };
    auto dot = [&](const cf32x4(&g)[NCH], const cf32x4(&w)[NCH]) __attribute__((always_inline)) -> float {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const cf32x4 v = valid(g, c);
            // one fused multiply-add per element, two independent chains
            s0 = fmaf(v.x, w[c].x, s0);
            s1 = fmaf(v.z, w[c].z, s1);
            s0 = fmaf(v.y, w[c].y, s0);
            s1 = fmaf(v.w, w[c].w, s1);
        }
        return block_sum(s0 + s1);
    };

    cf32x4 w[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) w[c] = cf32x4{0.f, 0.f, 0.f, 0.f};

    // ---- initial lists, counters, and w for a warm start
    for (int t = gl; t < np; t += T) { st_wg(&lb[o_act + t], int32_t(t)); st_wg(&cnt[t], uint8_t(0)); }
    // w = sum_t alpha_t y_t g_t over the non-zero alpha, compensated (Kahan) summation in fp32:
    // used for a warm start and to shed the rounding drift of the incremental updates before
    // the stopping rule is verified.  Returns the number of rows read.
    auto recompute_w = [&]() __attribute__((always_inline)) -> int {
        cf32x4 comp[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c) { w[c] = cf32x4{0.f, 0.f, 0.f, 0.f}; comp[c] = cf32x4{0.f, 0.f, 0.f, 0.f}; }
        int used = 0;
        for (int b0 = 0; b0 < np; b0 += 64) {
            // every wavefront scans the same 64 values and adds the rows of the non-zero ones
            const int t0 = b0 + (gl & 63);
            const float av = t0 < np ? ld_wg(&alpha[t0]) : 0.0f;
            unsigned long long todo = __ballot(av != 0.0f);
            while (todo) {
                // up to D rows requested together, then added in index order
                cf32x4 g[D][NCH];
                float f[D];
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    f[u] = 0.0f;
                    if (todo) {
                        const int j = __ffsll(todo) - 1;
                        todo &= todo - 1;
                        load_row(g[u], row_of(b0 + j));
                        f[u] = __shfl(av, j, 64) * y[b0 + j];
                        ++used;
                    }
                }
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    if (f[u] != 0.0f) {
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            const cf32x4 term = f[u] * valid(g[u], c) - comp[c];
                            const cf32x4 sum = w[c] + term;
                            comp[c] = (sum - w[c]) - term;
                            w[c] = sum;
                        }
                    }
                }
            }
        }
        return used;
    };
    wg_sync();
    recompute_w();
    wg_sync();

    int n_act = np, n_rem = 0, head = 0, since = 0, epochs = 0, converged = 0, fresh = 1;   // the start w is computed from alpha
    int64_t steps = 0;
    float maxviol = 0.f;

    // one step on a removed variable (re-check) or a violation probe; slow path, no prefetch
    auto single = [&](int t, bool apply, float &viol_out) __attribute__((always_inline)) -> bool {
        const int64_t row = row_of(t);
        const float yt = y[t];
        const float at = ld_wg(&alpha[t]);
        const float q = a.gsq[row];
        cf32x4 g[NCH];
        load_row(g, row);
        const float grad = 1.0f - yt * dot(g, w);
        viol_out = cd_violation(at, grad, C);
        if (!apply) return false;
        float an = q > 0.0f ? at + grad / q : C;
        an = fminf(fmaxf(an, 0.0f), C);
        if (an != at) {
            const float dl = (an - at) * yt;
#pragma unroll
            for (int c = 0; c < NCH; ++c) w[c] += dl * valid(g, c);
            if (gl == 0) st_wg(&alpha[t], an);
            return true;
        }
        return false;
    };

    while (epochs < a.max_epochs && !converged) {
        int n_nxt = 0;
        maxviol = 0.f;
        for (int b0 = 0; b0 < n_act; b0 += BLK) {
            const int nb = min(BLK, n_act - b0);
            // gather the metadata of the next nb steps, one step per lane
            wg_sync();
            if (gl < nb) {
                const int t = ld_wg(&lb[o_act + b0 + gl]);
                const int64_t row = row_of(t);
                s_t[gl] = t;
                s_row[gl] = row;
                s_y[gl] = y[t];
                s_alpha[gl] = ld_wg(&alpha[t]);
                s_cnt[gl] = ld_wg(&cnt[t]);
                const float qq = a.gsq[row];
                s_q[gl] = qq > 0.0f ? 1.0f / qq : 0.0f;     // reciprocal, off the steps' dependent path
            }
            __syncthreads();
            // ring of D row buffers: the row of step j + D - 1 is requested at step j, so D - 1 row
            // loads are in flight behind the one being consumed (a step is far shorter than a trip
            // to memory)
            cf32x4 gr[D][NCH];
#pragma unroll
            for (int u = 0; u < D - 1; ++u) load_row(gr[u], s_row[min(u, nb - 1)]);
            auto step = [&](int j, const cf32x4(&g)[NCH], cf32x4(&gn)[NCH]) __attribute__((always_inline)) {
                // the eta share: one step on the head of the removed queue
                if (a.shrink_k > 0 && a.check_every > 0 && since >= a.check_every && n_rem > 0) {
                    wg_sync();              // the lists are written by one lane: make its stores visible
                    const int t = ld_wg(&lb[o_rem + head]);
                    head = head + 1 == cap ? 0 : head + 1;
                    --n_rem;
                    float v;
                    const bool changed = single(t, true, v);
                    ++steps;
                    since = 0;
                    int tail = head + n_rem;
                    if (tail >= cap) tail -= cap;
                    const int64_t slot = changed ? o_nxt + n_nxt : o_rem + tail;
                    if (gl == 0) {
                        if (changed) st_wg(&cnt[t], uint8_t(0));
                        st_wg(&lb[slot], int32_t(t));
                    }
                    const int ch = changed ? 1 : 0;
                    n_nxt += ch;
                    n_rem += 1 - ch;
                }
                // into the buffer step j-1 released.  Unconditional (past the end of the block the last row
                // is fetched again and never used): a branch around the loads would merge a path without
                // them into the wait counts, and every step would then wait for its own prefetch
                load_row(gn, s_row[min(j + D - 1, nb - 1)]);
                const int t = s_t[j];
                const float yt = s_y[j], at = s_alpha[j], qinv = s_q[j];
                const float grad = 1.0f - yt * dot(g, w);            // step 2a
                maxviol = fmaxf(maxviol, cd_violation(at, grad, C));
                float an = qinv > 0.0f ? at + grad * qinv : C;       // step 2b
                an = fminf(fmaxf(an, 0.0f), C);
                ++steps;
                ++since;
                // the same instructions whatever the outcome (a zero update of w, the same three
                // stores), so that loads in flight are never waited for because of a branch
                const bool changed = an != at;
                const float dl = (an - at) * yt;
#pragma unroll
                for (int c = 0; c < NCH; ++c) w[c] += dl * valid(g, c);
                const int cn = changed ? 0 : s_cnt[j] + 1;
                const bool drop = !changed && a.shrink_k > 0 && cn >= a.shrink_k;
                int tail = head + n_rem;
                if (tail >= cap) tail -= cap;
                const int64_t slot = drop ? o_rem + tail : o_nxt + n_nxt;
                if (gl == 0) {
                    st_wg(&alpha[t], an);
                    st_wg(&cnt[t], uint8_t(cn));
                    st_wg(&lb[slot], int32_t(t));
                }
                const int dr = drop ? 1 : 0;
                n_rem += dr;
                n_nxt += 1 - dr;
            };
            // whole groups of D steps run without a guard between them (a guard is a branch, and a branch
            // between a prefetch and its use costs the overlap, as above); the ragged end of the last
            // block of an epoch takes the guarded form
            int j0 = 0;
            for (; j0 + D <= nb; j0 += D) {
#pragma unroll
                for (int u = 0; u < D; ++u) step(j0 + u, gr[u], gr[(u + D - 1) % D]);
            }
            if (j0 < nb) {
#pragma unroll
                for (int u = 0; u < D; ++u)
                    if (j0 + u < nb) step(j0 + u, gr[u], gr[(u + D - 1) % D]);
            }
        }
        ++epochs;
        if (maxviol <= a.eps) {
            // recompute w from alpha, then sweep over the removed variables with w fixed
            wg_sync();
            steps += recompute_w();
            int back = 0, kept = 0;
            const int m = n_rem;
            const int head0 = head;
            for (int b0 = 0; b0 < m; b0 += BLK) {
                const int nb = min(BLK, m - b0);
                wg_sync();
                if (gl < nb) {
                    int at_ = head0 + b0 + gl;
                    if (at_ >= cap) at_ -= cap;
                    const int t = ld_wg(&lb[o_rem + at_]);
                    s_t[gl] = t;
                    s_row[gl] = row_of(t);
                    s_y[gl] = y[t];
                    s_alpha[gl] = ld_wg(&alpha[t]);
                }
                __syncthreads();
                for (int j0 = 0; j0 < nb; j0 += D) {
                    // D independent rows: loads, partial sums and reductions overlap
                    cf32x4 g[D][NCH];
                    float f[D];
#pragma unroll
                    for (int u = 0; u < D; ++u)
                        if (j0 + u < nb) load_row(g[u], s_row[j0 + u]);
#pragma unroll
                    for (int u = 0; u < D; ++u) f[u] = j0 + u < nb ? dot(g[u], w) : 0.0f;
#pragma unroll
                    for (int u = 0; u < D; ++u) {
                        if (j0 + u < nb) {
                            const int t = s_t[j0 + u];
                            const float grad = 1.0f - s_y[j0 + u] * f[u];
                            ++steps;
                            const bool viol = cd_violation(s_alpha[j0 + u], grad, C) > a.eps;
                            // kept entries are rewritten behind the old tail, in order; that region
                            // only ever overlaps entries of the ring that were already consumed
                            int tail = head0 + m + kept;
                            if (tail >= cap) tail -= cap;
                            if (tail >= cap) tail -= cap;
                            const int64_t slot = viol ? o_nxt + n_nxt : o_rem + tail;
                            if (gl == 0) {
                                if (viol) st_wg(&cnt[t], uint8_t(0));
                                st_wg(&lb[slot], int32_t(t));
                            }
                            const int vi = viol ? 1 : 0;
                            n_nxt += vi;
                            back += vi;
                            kept += 1 - vi;
                        }
                    }
                }
            }
            head = head0 + m;
            if (head >= cap) head -= cap;
            n_rem = kept;
            if (back == 0 && fresh) converged = 1;      // this epoch already started from a recomputed w
            fresh = 1;
        } else {
            fresh = 0;
        }
        o_act = (epochs & 1) ? stride : 0;
        o_nxt = stride - o_act;
        n_act = n_nxt;
    }

    // ---- results: w, dual objective, status
    wg_sync();
    float ww = 0.f, sa = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        ww += w[c].x * w[c].x + w[c].y * w[c].y + w[c].z * w[c].z + w[c].w * w[c].w;
        const int col = (c * T + gl) * 4;
        float *wo = a.w + int64_t(p) * a.ldw + col;
        if (col < r) wo[0] = w[c].x;
        if (col + 1 < r) wo[1] = w[c].y;
        if (col + 2 < r) wo[2] = w[c].z;
        if (col + 3 < r) wo[3] = w[c].w;
    }
    for (int t = gl; t < np; t += T) sa += ld_wg(&alpha[t]);
    ww = block_sum(ww);
    sa = block_sum(sa);
    if (gl == 0) {
        CdStatus st;
        st.steps = steps;
        st.epochs = epochs;
        st.converged = converged;
        st.active = n_act;
        st.max_violation = maxviol;
        st.dual = sa - 0.5f * ww;
        st.reserved = 0;
        a.status[p] = st;
    }
}

}  // namespace lpd
