// fp32 MFMA GEMM for gfx950:  C[M x N] = epilogue( A[M x K] * B[N x K]^T ).
//
// Both operands are row-major and contracted over their contiguous axis, which
// is the shape of both products of Figure 1 step 1d: the distance contraction
// X L^T (contraction over the d features) and the whitening product Z W^T
// (contraction over the B landmarks).
//
// Design for CDNA4:
//   * one workgroup = WGM x WGN wavefronts of 64 lanes, each wavefront owns a
//     (BM/WGM) x (BN/WGN) block of C as 32x32 accumulator tiles of
//     v_mfma_f32_32x32x2_f32 (lane l feeds A[row l%32][k l/32] and
//     B[col l%32][k l/32]; accumulator register v of lane l is
//     C[8*(v/4) + 4*(l/32) + v%4][l%32]).
//   * global -> registers -> LDS with 16-byte accesses, double-buffered LDS,
//     one barrier per k-tile.  LDS rows keep the k index contiguous
//     ([row][BK+4] floats): the +4 pad makes the 16-byte reads of 16 consecutive
//     rows hit 16 distinct bank groups.  Each lane reads 4 consecutive k with
//     one ds_read_b128; lanes 0-31 take k0..k0+3 and lanes 32-63 k0+4..k0+7, so
//     the 4 MFMA steps of a read pair k = (k0+t, k0+4+t).  A and B use the same
//     pairing, and a sum does not care in which order k is visited.
//     (Loading tiles straight into LDS, global_load_lds_dwordx4 into unpadded XOR-swizzled
//     stages, was built and measured: bit-identical results, 146.6 against 150.2 TFLOP/s on the
//     256x256 tile whether 2, 3 or 4 stages were in flight, so the loads go through registers.)
//   * workgroup ids are remapped so that the ids one XCD receives (id mod 8)
//     form a contiguous range of tiles, and tiles are walked in groups of GM
//     tile rows, so the 32 workgroups resident on an XCD share A and B strips
//     in that XCD's L2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace lpd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int I>
using SI = std::integral_constant<int, I>;

enum { EPI_STORE = 0, EPI_GAUSS = 1, EPI_GAUSS_DOT = 2 };
constexpr int GEMM_DOT_MAX = 64;     // weight vectors the EPI_GAUSS_DOT write-out takes at once
constexpr int GEMM_DOT_FMA_MAX = 6;  // up to here the write-out multiplies by them with vector FMAs, above on the MFMA units

struct GemmArgs {
    const float *A;  // M x K
    const float *B;  // N x K
    float *C;        // M x n_store
    int64_t lda, ldb, ldc;
    int M, N, K;
    int n_store;     // columns [N, n_store) of C are written as zeros
    int tiles_m, tiles_n;
    // EPI_GAUSS: C = exp2(scale * max(0, na[row] + nb[col] - 2 acc)), scale = -gamma * log2(e).
    // Both operands are read as A[i,k] - cen[k], B[j,k] - cen[k] (cen: K floats, 16-byte aligned) and
    // na, nb are the squared norms of the shifted rows: a distance does not depend on the origin, and
    // with the origin inside the data the three terms of the expansion are of the size of the
    // distance itself instead of the size of ||x||^2, which is what their fp32 rounding scales with.
    const float *na, *nb, *cen;
    float scale;
    // EPI_GAUSS_DOT: the kernel block is not written; its tile is multiplied at once by nv <= GEMM_DOT_MAX weight
    // vectors (rows of V, nv x N, leading dimension ldv) and the tile's share of the scores goes to
    // P[tile column][row][vector] (tiles_n x M x nv floats); a pass over the tile columns adds them up.
    const float *V;
    int64_t ldv;
    int nv;
    float *P;
};

constexpr int GEMM_BK = 16;
constexpr int GEMM_LDK = GEMM_BK + 4;

// two stages of operand tiles, then the BM + BN squared norms of the tile's rows and columns (EPI_GAUSS),
// then the tile's columns of the weight vectors (EPI_GAUSS_DOT)
// (nv: the weight vectors of the launch; their slots are the last thing in LDS, so a launch with fewer asks for less)
template <int BM, int BN, int EPI = EPI_STORE>
constexpr size_t gemm_lds_bytes(int nv = GEMM_DOT_MAX)
{
    return (size_t(2) * (BM + BN) * GEMM_LDK + (BM + BN) + (EPI == EPI_GAUSS_DOT ? nv * (BN + 4) : 0)) * sizeof(float);
}

template <int BM, int BN, int WGM, int WGN, bool ALIGNED, int EPI, int PIPE>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_nt_kernel(GemmArgs p)
{
    constexpr int BK = GEMM_BK, LDK = GEMM_LDK;
    constexpr bool GAUSS = EPI != EPI_STORE;      // the kernel block, written out (EPI_GAUSS) or contracted at once (EPI_GAUSS_DOT)
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CPR = BK / 4;        // 16-byte chunks per tile row
    constexpr int RPP = NT / CPR;      // tile rows filled per pass of the workgroup
    constexpr int PA = BM / RPP, PB = BN >= RPP ? BN / RPP : 1;
    constexpr bool BPART = BN < RPP;   // a narrow tile: only the first BN loader rows carry rows of B (whole wavefronts: 16 rows each)
    constexpr int STAGE = (BM + BN) * LDK;
    static_assert(BM % RPP == 0 && (BN % RPP == 0 || (BN < RPP && BN % 16 == 0)), "tile rows must be a multiple of the loader pass");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");

    extern __shared__ __attribute__((aligned(16))) float lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- workgroup id -> tile, XCD-aware and grouped
    int tm, tn;
    {
        const int nwg = gridDim.x;
        const int id = blockIdx.x;
        const int per = nwg >> 3;
        const int lin = (id < (per << 3)) ? (id & 7) * per + (id >> 3) : id;
        constexpr int GM = 8;
        const int group_sz = GM * p.tiles_n;
        const int g = lin / group_sz;
        const int first_m = g * GM;
        const int gm = min(p.tiles_m - first_m, GM);
        const int within = lin - g * group_sz;
        tm = first_m + within % gm;
        tn = within / gm;
    }
    const int m0 = tm * BM, n0 = tn * BN;

    // Tiles that lie entirely in the zero-filled columns do no arithmetic.
    if (EPI == EPI_STORE && n0 >= p.N) {
        for (int e = tid; e < BM * BN; e += NT) {
            const int rr = m0 + e / BN, cc = n0 + e % BN;
            if (rr < p.M && cc < p.n_store) p.C[int64_t(rr) * p.ldc + cc] = 0.0f;
        }
        return;
    }

    // ---- global loader set-up: thread -> (row within pass, 16-byte chunk)
    const int lrow = tid / CPR, lch = tid % CPR;
    const float *ga[PA], *gb[PB];
#pragma unroll
    for (int q = 0; q < PA; ++q) {
        const int rr = min(m0 + lrow + q * RPP, p.M - 1);
        ga[q] = p.A + int64_t(rr) * p.lda + lch * 4;
    }
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int rr = min(n0 + lrow + q * RPP, p.N - 1);
        gb[q] = p.B + int64_t(rr) * p.ldb + lch * 4;
    }

    // rc: the four centre values of this thread's k columns (all its rows share them).  They are loaded with
    // the tile and subtracted on the way into LDS, so that nothing waits for a global load before it must.
    constexpr int NSET = PIPE == 2 ? 2 : PIPE == 4 ? 4 : 1;   // register sets of staged tiles (see the pipelined schedule)
    f32x4 ra_[NSET][PA], rb_[NSET][PB], rc_[NSET];
    f32x4(&ra)[PA] = ra_[0];
    f32x4(&rb)[PB] = rb_[0];
    f32x4 &rc = rc_[0];
    rc = f32x4{0.f, 0.f, 0.f, 0.f};
    auto gload = [&](int k0) {
        const int k = k0 + lch * 4;
        if (ALIGNED) {
            if (k < p.K) {
#pragma unroll
                for (int q = 0; q < PA; ++q) ra[q] = *reinterpret_cast<const f32x4 *>(ga[q] + k0);
#pragma unroll
                for (int q = 0; q < PB; ++q) rb[q] = *reinterpret_cast<const f32x4 *>(gb[q] + k0);
                if (GAUSS) rc = *reinterpret_cast<const f32x4 *>(p.cen + k);
            } else {
#pragma unroll
                for (int q = 0; q < PA; ++q) ra[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < PB; ++q) rb[q] = f32x4{0.f, 0.f, 0.f, 0.f};
                rc = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        } else {
#pragma unroll
            for (int q = 0; q < PA; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) ra[q][e] = (k + e < p.K) ? ga[q][k0 + e] : 0.0f;
#pragma unroll
            for (int q = 0; q < PB; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) rb[q][e] = (k + e < p.K) ? gb[q][k0 + e] : 0.0f;
            if (GAUSS) {
#pragma unroll
                for (int e = 0; e < 4; ++e) rc[e] = (k + e < p.K) ? p.cen[k + e] : 0.0f;
            }
        }
    };
    auto lstore = [&](int buf) {
        float *As = lds + buf * STAGE;
        float *Bs = As + BM * LDK;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            *reinterpret_cast<f32x4 *>(&As[(lrow + q * RPP) * LDK + lch * 4]) = GAUSS ? ra[q] - rc : ra[q];
#pragma unroll
        for (int q = 0; q < PB; ++q)
            if (!BPART || lrow < BN)
                *reinterpret_cast<f32x4 *>(&Bs[(lrow + q * RPP) * LDK + lch * 4]) = GAUSS ? rb[q] - rc : rb[q];
    };

    // The squared norms the epilogue needs go to LDS now, so that after the main loop nothing waits for
    // global memory: a load there would also wait for every store issued before it (one counter orders both).
    float *nas = lds + 2 * STAGE, *nbs = nas + BM;
    if (GAUSS) {
        for (int e = tid; e < BM + BN; e += NT)
            nas[e] = e < BM ? p.na[min(m0 + e, p.M - 1)] : p.nb[min(n0 + e - BM, p.N - 1)];
    }
    // EPI_GAUSS_DOT: the tile's columns of the weight vectors, zero past column N, so that a column outside the
    // matrix adds nothing whatever its accumulator holds
    // (whole groups of 32 vectors, zero past the last one; rows padded like the operand stages: the write-out reads
    // them as MFMA operand fragments)
    constexpr int VLD = BN + 4;
    float *vs = nbs + BN;
    if constexpr (EPI == EPI_GAUSS_DOT) {
        const int nvpad = (p.nv + 31) / 32 * 32;
        for (int e = tid; e < nvpad * BN; e += NT) {
            const int q = e / BN, cl = e - q * BN;
            vs[q * VLD + cl] = q < p.nv && n0 + cl < p.N ? p.V[int64_t(q) * p.ldv + n0 + cl] : 0.0f;
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int frag_row = lane & 31;
    const int frag_k = (lane >> 5) * 4;
    const int a_off = (wm * WM + frag_row) * LDK + frag_k;
    const int b_off = BM * LDK + (wn * WN + frag_row) * LDK + frag_k;

    const int nk = (p.K + BK - 1) / BK;

    if constexpr (PIPE == 0) {
        // Plain schedule: load next tile, compute the current one, store, barrier.
        gload(0);
        lstore(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            const bool more = kt + 1 < nk;
            if (more) gload((kt + 1) * BK);

            const float *S = lds + cur * STAGE;
#pragma unroll
            for (int kc = 0; kc < BK / 8; ++kc) {
                f32x4 a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = *reinterpret_cast<const f32x4 *>(&S[a_off + i * 32 * LDK + kc * 8]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = *reinterpret_cast<const f32x4 *>(&S[b_off + j * 32 * LDK + kc * 8]);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[j][t], acc[i][j], 0, 0, 0);
            }

            if (more) lstore(cur ^ 1);
            __syncthreads();
        }
    } else {
        // Software-pipelined schedule for the aligned fast path (BK = 16 = two 8-k chunks per tile).
        //
        //   phase A  MFMA chunk 0 of tile kt | fetch chunk-1 fragments | staged registers (tile kt+1) -> LDS
        //   barrier
        //   phase B  MFMA chunk 1 of tile kt | global loads of tile kt+2 | fetch chunk-0 fragments of tile kt+1
        //
        // The barrier sits between the chunks and fragments are fetched one chunk ahead, across it,
        // so a wavefront always has MFMAs queued while LDS, global memory or the other wavefronts
        // catch up.  A wavefront issues in order: a burst of LDS or global instructions that fills
        // the memory queues would hold back the MFMAs behind it, so the scheduler is told to place
        // one memory instruction per MPG MFMAs.  The loop body is branch-free: tiles past the last
        // full one are redirected to the last full one (redundant, in-bounds, unused), global
        // addresses are a wave-uniform base plus a per-lane 32-bit byte offset fixed before the loop.
        // Buffer (kt+1)&1 is overwritten in phase A of iteration kt; its previous tile kt-1 was last
        // read before the barrier of iteration kt-1, and each wavefront drains its LDS reads before a
        // barrier.  A partial last tile (K % 16 != 0) is handled after the loop by the plain schedule.
        static_assert(PIPE == 1 || PIPE == 2 || PIPE == 4,
                      "schedules: 0 plain, 1 pipelined, 2 and 4 pipelined with that many staged tiles");
        static_assert(BK == 16, "the pipelined schedule assumes two chunks per tile");
        static_assert(ALIGNED, "the pipelined schedule is for the 16-byte aligned fast path");
        constexpr int MEMOPS = TM + TN + PA + PB + (GAUSS ? 1 : 0);   // + the load of the centre values
        constexpr int MPG = (4 * TM * TN) / MEMOPS > 0 ? (4 * TM * TN) / MEMOPS : 1;
        constexpr bool WRITES_FIRST = NSET >= 2;
        const int nfull = p.K / BK;

        if (nfull > 0) {
            const char *baseA = reinterpret_cast<const char *>(p.A + int64_t(m0) * p.lda);
            const char *baseB = reinterpret_cast<const char *>(p.B + int64_t(n0) * p.ldb);
            uint32_t oa[PA], ob[PB];
#pragma unroll
            for (int q = 0; q < PA; ++q)
                oa[q] = uint32_t(min(lrow + q * RPP, p.M - 1 - m0)) * uint32_t(p.lda) * 4u + lch * 16u;
#pragma unroll
            for (int q = 0; q < PB; ++q)
                ob[q] = uint32_t(min(lrow + q * RPP, p.N - 1 - n0)) * uint32_t(p.ldb) * 4u + lch * 16u;
            auto gload_full = [&](int tile, auto S) {
                constexpr int st = decltype(S)::value;
                const char *pa = baseA + size_t(tile) * (BK * 4);
                const char *pb = baseB + size_t(tile) * (BK * 4);
#pragma unroll
                for (int q = 0; q < PA; ++q) ra_[st][q] = *reinterpret_cast<const f32x4 *>(pa + oa[q]);
#pragma unroll
                for (int q = 0; q < PB; ++q) rb_[st][q] = *reinterpret_cast<const f32x4 *>(pb + ob[q]);
                if (GAUSS) rc_[st] = *reinterpret_cast<const f32x4 *>(p.cen + tile * BK + lch * 4);
            };
            // Two consecutive k-tiles at once, into sets S0 and S1: a row's 64 bytes of an even tile and of the odd
            // tile behind it are the two halves of one 128-byte line (rows aligned to that), and asking for both
            // in the same breath is what keeps the line from being fetched twice (see the four-set schedule).
            auto gload_pair = [&](int tile0, int tile1, auto S0, auto S1) {
                constexpr int s0 = decltype(S0)::value, s1 = decltype(S1)::value;
                const char *pa0 = baseA + size_t(tile0) * (BK * 4), *pa1 = baseA + size_t(tile1) * (BK * 4);
                const char *pb0 = baseB + size_t(tile0) * (BK * 4), *pb1 = baseB + size_t(tile1) * (BK * 4);
#pragma unroll
                for (int q = 0; q < PA; ++q) {
                    ra_[s0][q] = *reinterpret_cast<const f32x4 *>(pa0 + oa[q]);
                    ra_[s1][q] = *reinterpret_cast<const f32x4 *>(pa1 + oa[q]);
                }
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    rb_[s0][q] = *reinterpret_cast<const f32x4 *>(pb0 + ob[q]);
                    rb_[s1][q] = *reinterpret_cast<const f32x4 *>(pb1 + ob[q]);
                }
                if (GAUSS) {
                    rc_[s0] = *reinterpret_cast<const f32x4 *>(p.cen + tile0 * BK + lch * 4);
                    rc_[s1] = *reinterpret_cast<const f32x4 *>(p.cen + tile1 * BK + lch * 4);
                }
            };
            auto lstore_set = [&](int buf, auto S) {
                constexpr int st = decltype(S)::value;
                float *As = lds + buf * STAGE;
                float *Bs = As + BM * LDK;
#pragma unroll
                for (int q = 0; q < PA; ++q)
                    *reinterpret_cast<f32x4 *>(&As[(lrow + q * RPP) * LDK + lch * 4]) =
                        GAUSS ? ra_[st][q] - rc_[st] : ra_[st][q];
#pragma unroll
                for (int q = 0; q < PB; ++q)
                    if (!BPART || lrow < BN)
                        *reinterpret_cast<f32x4 *>(&Bs[(lrow + q * RPP) * LDK + lch * 4]) =
                            GAUSS ? rb_[st][q] - rc_[st] : rb_[st][q];
            };
            f32x4 a0[TM], b0[TN], a1[TM], b1[TN];
            auto fetch = [&](f32x4(&a)[TM], f32x4(&b)[TN], int buf, int kc) {
                const float *S = lds + buf * STAGE;
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = *reinterpret_cast<const f32x4 *>(&S[a_off + i * 32 * LDK + kc * 8]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = *reinterpret_cast<const f32x4 *>(&S[b_off + j * 32 * LDK + kc * 8]);
            };
            auto mma = [&](const f32x4(&a)[TM], const f32x4(&b)[TN]) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[j][t], acc[i][j], 0, 0, 0);
            };
            // One k-tile.  Register set S holds tile kt+1 on entry and is refilled with tile kt+1+NSET, so with
            // two sets a global load has a whole iteration and a half to arrive instead of half of one: what
            // streams from HBM rather than from L2 (W of many landmarks) then never holds up phase A.  (A third
            // set measured no faster on the 256x256 tile, whose registers it overflows.)
            // Four sets, for the narrow tiles (at most 64 columns against the rows of a matrix far larger than the
            // caches, read once): more tiles in flight buy nothing by themselves, but a row's 64 bytes of an even
            // and of the following odd k-tile are one 128-byte line, and with some 200,000 rows in flight on the
            // chip the L2s lose the line between two separate visits (a third more bytes fetched than the matrix
            // holds).  So the two are requested together, every other step.
            // LD: k-tiles requested in this step.  1 with one or two sets; with four sets 2 and 0 in turn: an even step
            // requests tiles kt+4 and kt+5 together, into the set the previous step emptied and the one this step
            // empties.
            auto step = [&](int kt, auto S, auto LD) {
                constexpr int nld = decltype(LD)::value;
                constexpr int st = decltype(S)::value;
                const int cur = kt & 1;
                // ---- phase A
                // (program order matters too: the compiler keeps LDS reads and writes it cannot tell apart in it)
                if constexpr (WRITES_FIRST) lstore_set(cur ^ 1, S);
                fetch(a1, b1, cur, 1);
                mma(a0, b0);
                if constexpr (!WRITES_FIRST) lstore_set(cur ^ 1, S);
                // A wavefront drains its LDS traffic before the barrier and issues nothing meanwhile, so what
                // it issued last should be long done by then: the writes go first where the staged tile has
                // had time to arrive (two sets), the reads first where it may not have (one set).
                if constexpr (WRITES_FIRST) {
#pragma unroll
                    for (int g = 0; g < PA + PB; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // one LDS write
                        __builtin_amdgcn_sched_group_barrier(0x008, MPG, 0); // MPG MFMAs
                    }
                }
#pragma unroll
                for (int g = 0; g < TM + TN; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                    __builtin_amdgcn_sched_group_barrier(0x008, MPG, 0);
                }
                if constexpr (!WRITES_FIRST) {
#pragma unroll
                    for (int g = 0; g < PA + PB; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, MPG, 0);
                    }
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4 * TM * TN - MPG * (TM + TN + PA + PB), 0);   // the rest of the MFMAs
                __builtin_amdgcn_sched_barrier(0);      // each phase is scheduled on its own
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                // ---- phase B
                if constexpr (nld == 1) gload_full(min(kt + 1 + NSET, nfull - 1), S);
                if constexpr (nld == 2)
                    gload_pair(min(kt + NSET, nfull - 1), min(kt + 1 + NSET, nfull - 1), SI<(st + NSET - 1) % NSET>{}, S);
                fetch(a0, b0, cur ^ 1, 0);
                mma(a1, b1);
                constexpr int LOADGROUPS = nld == 0 ? 0 : PA + PB + (GAUSS ? 1 : 0);
#pragma unroll
                for (int g = 0; g < LOADGROUPS; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x020, nld, 0);   // one global load (a pair with four sets)
                    __builtin_amdgcn_sched_group_barrier(0x008, MPG, 0);
                }
#pragma unroll
                for (int g = 0; g < TM + TN; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, MPG, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4 * TM * TN - MPG * (TM + TN + LOADGROUPS), 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            // tile j of the contraction travels in register set j % NSET
            using LD_EVEN = SI<NSET == 4 ? 2 : 1>;
            using LD_ODD = SI<NSET == 4 ? 0 : 1>;
            gload_full(0, SI<0>{});
            lstore_set(0, SI<0>{});
            gload_full(min(1, nfull - 1), SI<1 % NSET>{});
            if constexpr (NSET > 1) gload_full(min(2, nfull - 1), SI<2 % NSET>{});
            if constexpr (NSET > 2) gload_full(min(3, nfull - 1), SI<3 % NSET>{});
            __syncthreads();
            fetch(a0, b0, 0, 0);

            int kt = 0;
            for (; kt + NSET <= nfull; kt += NSET) {
                step(kt, SI<1 % NSET>{}, LD_EVEN{});
                if constexpr (NSET > 1) step(kt + 1, SI<2 % NSET>{}, LD_ODD{});
                if constexpr (NSET > 2) step(kt + 2, SI<3 % NSET>{}, LD_EVEN{});
                if constexpr (NSET > 3) step(kt + 3, SI<4 % NSET>{}, LD_ODD{});
            }
            // (kt is a multiple of NSET here: tile kt+1+i sits in set (i+1) % NSET)
            if constexpr (NSET > 1) {
                if (kt < nfull) step(kt++, SI<1 % NSET>{}, LD_EVEN{});
            }
            if constexpr (NSET > 2) {
                if (kt < nfull) step(kt++, SI<2 % NSET>{}, LD_ODD{});
            }
            if constexpr (NSET > 3) {
                if (kt < nfull) step(kt++, SI<3 % NSET>{}, LD_EVEN{});
            }
            __syncthreads();
        }
        if (nfull < nk) {
            // partial last tile, zero-filled past K
            gload(nfull * BK);
            lstore(0);
            __syncthreads();
            const float *S = lds;
#pragma unroll
            for (int kc = 0; kc < BK / 8; ++kc) {
                f32x4 a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = *reinterpret_cast<const f32x4 *>(&S[a_off + i * 32 * LDK + kc * 8]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = *reinterpret_cast<const f32x4 *>(&S[b_off + j * 32 * LDK + kc * 8]);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[j][t], acc[i][j], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: accumulator register v of lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32]
    const int col_in = lane & 31;
    const int row_in = (lane >> 5) * 4;
    if (GAUSS) __syncthreads();      // the norms in LDS (no barrier lies behind when K = 0)
    auto finish = [&](float accv, float nav, float nbv) __attribute__((always_inline)) -> float {
        if (!GAUSS) return accv;
        const float dist = fmaxf(nav + nbv - 2.0f * accv, 0.0f);
        return __builtin_amdgcn_exp2f(p.scale * dist);
    };
    if constexpr (EPI == EPI_GAUSS_DOT) {
        // Scores of the tile's rows against nv weight vectors, straight from the accumulators (prediction, Section 4
        // "Algorithm Overview": K(x, L) times the folded weights; the kernel block never leaves the chip).
        //   1. z in place of the accumulators (rows past M are never written out, columns past N meet zero weights);
        //   2. a wavefront's scores F_w = z_w V_w^T, its WM x WN block of z against its WN columns of the weight
        //      vectors, on the MFMA units: 32 vectors at a time fill the output columns of a 32x32 tile.  z is in
        //      accumulator layout (a lane holds one column), the A operand wants a lane to hold one row, so each
        //      32x32 block of z passes through a patch of LDS that belongs to its wavefront alone (LDS serves a
        //      wavefront's accesses in the order it issued them: no barrier, no wait);
        //   3. the WGN wavefronts side by side hold shares of the same rows: the right one hands its share over
        //      through LDS, the left one adds and writes the tile's BM x nv scores to P.  No atomics: the order of
        //      every sum is fixed.
        static_assert(WGN <= 2, "two wavefronts across at most");
        constexpr int NVG = GEMM_DOT_MAX / 32;             // groups of 32 weight vectors
        constexpr int PLD = 32 + 4;                        // patch rows padded like the operand stages
        constexpr int FLD = GEMM_DOT_MAX + 1;
        static_assert(WGM * WGN * 32 * PLD <= 2 * STAGE && BM * FLD <= 2 * STAGE,
                      "patches and handed-over scores take the place of the operand stages");
        const int ngr = (p.nv + 31) / 32;
        float nbv[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) nbv[j] = nbs[wn * WN + j * 32 + col_in];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float nav = nas[wm * WM + i * 32 + 8 * (v >> 2) + row_in + (v & 3)];
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j][v] = finish(acc[i][j][v], nav, nbv[j]);
            }
        __syncthreads();                                   // every wavefront is done with the operand stages
        if (p.nv <= GEMM_DOT_FMA_MAX) {
            // A handful of vectors: a 32-wide MFMA tile would be mostly padding and costs what ten vectors cost
            // this way.  Per vector: a lane's row slots times its TN columns, then a reduce-scatter over the 32
            // lanes that hold the same rows (after the five halving steps lane l holds the total of slot l), then
            // one LDS add per lane into the tile's scores (the WGN wavefronts side by side add into the same
            // entries: with at most two of them the sum does not depend on who comes first).
            constexpr int NSL = TM * 16;                  // row slots per lane: 32, or 16 for a wavefront of 32 rows
            static_assert(NSL == 32 || NSL == 16, "16 or 32 row slots per lane");
            float *ft = lds;                               // BM x FLD, over the operand stages
            for (int e = tid; e < BM * FLD; e += NT) ft[e] = 0.0f;
            __syncthreads();                               // ft is zero everywhere
            for (int q = 0; q < p.nv; ++q) {
                float vq[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) vq[j] = vs[q * VLD + wn * WN + j * 32 + col_in];
                float t[NSL];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float sum = 0.0f;
#pragma unroll
                        for (int j = 0; j < TN; ++j) sum += acc[i][j][v] * vq[j];
                        t[i * 16 + v] = sum;
                    }
                if constexpr (NSL == 16) {                     // 16 slots over 32 lanes: lanes l and l ^ 16 first join
#pragma unroll
                    for (int sl = 0; sl < 16; ++sl) t[sl] += __shfl_xor(t[sl], 16, 64);
                }
#pragma unroll
                for (int k = NSL / 2; k >= 1; k >>= 1) {
                    const bool up = (lane & k) != 0;           // this lane keeps the upper half of the slots
#pragma unroll
                    for (int sl = 0; sl < k; ++sl) {
                        // both slots are read into values first: a choice between two array elements would be turned
                        // into a per-lane index, and an array indexed per lane cannot live in registers
                        const float lo = t[sl], hi = t[sl + k];
                        const float keep = up ? hi : lo;
                        const float send = up ? lo : hi;
                        t[sl] = keep + __shfl_xor(send, k, 64);
                    }
                }
                // lane l now holds slot l % NSL = 16 i + v of its half-wavefront's rows (with 16 slots, twice over)
                const int sl = lane & (NSL - 1);
                const int rl = wm * WM + (sl >> 4) * 32 + 8 * ((sl & 15) >> 2) + row_in + (sl & 3);
                if (NSL == 32 || (lane & 16) == 0) atomicAdd(&ft[rl * FLD + q], t[0]);
            }
            __syncthreads();
            for (int e = tid; e < BM * p.nv; e += NT) {
                const int rl = e / p.nv, q = e - rl * p.nv;
                if (m0 + rl < p.M) p.P[(int64_t(tn) * p.M + m0 + rl) * p.nv + q] = ft[rl * FLD + q];
            }
            return;
        }
        // (two blocks at a time where two patches per wavefront fit: half as many waits for LDS)
        constexpr int NPB = (TN % 2 == 0 && 2 * WGM * WGN * 32 * PLD <= 2 * STAGE) ? 2 : 1;
        float *patch = lds + wave * (NPB * 32 * PLD);
        f32x16 fs[TM][NVG];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int g = 0; g < NVG; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) fs[i][g][v] = 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j0 = 0; j0 < TN; j0 += NPB) {
#pragma unroll
                for (int u = 0; u < NPB; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        patch[u * 32 * PLD + (8 * (v >> 2) + row_in + (v & 3)) * PLD + col_in] = acc[i][j0 + u][v];
                __builtin_amdgcn_s_waitcnt(0xc07f);        // lgkmcnt(0): the blocks are in LDS before they are read back
                __builtin_amdgcn_wave_barrier();           // (and the compiler keeps the reads behind the writes)
#pragma unroll
                for (int u = 0; u < NPB; ++u) {
#pragma unroll
                    for (int kc = 0; kc < 4; ++kc) {
                        const f32x4 za = *reinterpret_cast<const f32x4 *>(&patch[u * 32 * PLD + col_in * PLD + 8 * kc + row_in]);
#pragma unroll
                        for (int g = 0; g < NVG; ++g) {
                            if (g < ngr) {
                                const f32x4 vb = *reinterpret_cast<const f32x4 *>(
                                    &vs[(g * 32 + col_in) * VLD + wn * WN + (j0 + u) * 32 + 8 * kc + row_in]);
#pragma unroll
                                for (int t = 0; t < 4; ++t)
                                    fs[i][g] = __builtin_amdgcn_mfma_f32_32x32x2f32(za[t], vb[t], fs[i][g], 0, 0, 0);
                            }
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();           // (and the next blocks' writes behind these reads)
            }
        }
        // fs[i][g][v] is the score of row wm*WM + 32 i + 8 (v/4) + 4 (l/32) + v%4 against vector 32 g + l%32
        float *ft = lds;                                   // BM x FLD, over the patches
        if constexpr (WGN == 2) {
            __syncthreads();                               // all patches done with
            if (wn == 1) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int g = 0; g < NVG; ++g)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            ft[(wm * WM + i * 32 + 8 * (v >> 2) + row_in + (v & 3)) * FLD + g * 32 + col_in] = fs[i][g][v];
            }
            __syncthreads();
        }
        if (wn == 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int g = 0; g < NVG; ++g) {
                    const int q = g * 32 + col_in;
                    if (q >= p.nv) continue;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int rl = wm * WM + i * 32 + 8 * (v >> 2) + row_in + (v & 3);
                        float sum = fs[i][g][v];
                        if constexpr (WGN == 2) sum += ft[rl * FLD + q];
                        if (m0 + rl < p.M) p.P[(int64_t(tn) * p.M + m0 + rl) * p.nv + q] = sum;
                    }
                }
        }
    } else if (m0 + BM <= p.M && n0 + BN <= p.N) {
        // interior tile: no bounds to check, one row pointer per group of four rows
        float nbv[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) nbv[j] = GAUSS ? nbs[wn * WN + j * 32 + col_in] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int rl = wm * WM + i * 32 + 8 * g + row_in;      // row within the tile, a multiple of 4
                f32x4 nav = {0.f, 0.f, 0.f, 0.f};
                if (GAUSS) nav = *reinterpret_cast<const f32x4 *>(&nas[rl]);
                float *crow = p.C + int64_t(m0 + rl) * p.ldc + (n0 + wn * WN + col_in);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const float out = finish(acc[i][j][4 * g + e], nav[e], nbv[j]);
                        // G is not read again by this launch or the next: its stores need not stay in L2, where they
                        // would push out operand strips and leave dirty lines to write back when the kernel ends
                        if (EPI == EPI_STORE) __builtin_nontemporal_store(out, &crow[int64_t(e) * p.ldc + j * 32]);
                        else crow[int64_t(e) * p.ldc + j * 32] = out;
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int cl = wn * WN + j * 32 + col_in;
            const int cc = n0 + cl;
            if (cc >= p.n_store) continue;
            const bool live = cc < p.N;
            const float nbv = GAUSS ? nbs[cl] : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = wm * WM + i * 32 + 8 * (v >> 2) + row_in + (v & 3);
                    if (m0 + rl >= p.M) continue;
                    const float out = finish(acc[i][j][v], GAUSS ? nas[rl] : 0.0f, nbv);
                    if (EPI == EPI_STORE) __builtin_nontemporal_store(live ? out : 0.0f, &p.C[int64_t(m0 + rl) * p.ldc + cc]);
                    else p.C[int64_t(m0 + rl) * p.ldc + cc] = live ? out : 0.0f;
                }
            }
        }
    }
}

}  // namespace lpd
