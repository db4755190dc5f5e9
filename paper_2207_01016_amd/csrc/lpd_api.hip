// C ABI of the library (see include/lpd.h): argument checks, workspace
// carving, the row-panel schedule of Figure 1 step 1d, and kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

#include "../../include/lpd.h"
#include "cd_solver.hip.h"
#include "fused_small.hip.h"
#include "gemm_nt.hip.h"
#include "rowops.hip.h"
#include "whiten_internal.h"

// Scratch of lpd_predict_noalloc: one array per GPU, held from the first use of the library on that GPU until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels get the device
// address that call returns (static_scratch below), never the name.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace lpd;

constexpr int64_t kMaxDim = int64_t(1) << 30;   // n, d, B limits (32-bit tile arithmetic inside kernels)
constexpr size_t kAlign = 256;

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Leading dimension of the Z panel inside the workspace: a multiple of 4 floats
// (16-byte rows), nudged off large powers of two so the rows of one tile do not
// all start in the same memory channel.
inline int64_t panel_ld(int64_t B)
{
    int64_t ld = (B + 3) / 4 * 4;
    if (ld % 512 == 0) ld += 16;
    return ld;
}

struct Carve {
    size_t off_nx, off_nl, off_cen, off_z, min_bytes, rec_bytes;
    int64_t ldz, rec_rows, min_rows;
};

// norms of X (n), norms of L (B), the origin of the kernel block (d), then the Z panel
Carve carve(int64_t n, int64_t d, int64_t B)
{
    Carve c;
    c.ldz = panel_ld(B);
    c.off_nx = 0;
    c.off_nl = round_up(size_t(n) * 4, kAlign);
    c.off_cen = c.off_nl + round_up(size_t(B) * 4, kAlign);
    c.off_z = c.off_cen + round_up(size_t(d) * 4, kAlign);
    c.min_rows = std::min<int64_t>(n, 256);
    // recommended panel: about 32 Mi kernel values = 128 MB, half of the 256 MB Infinity Cache, so that a panel
    // written by the kernel-block launch can still be there when the whitening product reads it.  Rows =
    // 32 Mi / B rounded to 256 makes the 256x256 tile count of a panel a multiple of the 256 CUs whenever B is a
    // power of two (B >= 256): every round of workgroups of a launch is a full one (two rounds per launch).
    // Measured, ms per step at 16 / 32 / 64 / 128 Mi values: 7562 / 7498 / 7476 / 7477 (n = 2,000,000, B = 16,384),
    // 1509 / 1498 / 1497 (n = 1,280,000, B = 8,192; 32 Mi and up): flat from 32 Mi on, launches with fewer than 256
    // tiles (below 16 Mi) leave compute units idle.
    int64_t rows = (int64_t(32) << 20) / std::max<int64_t>(B, 1);
    rows = std::max<int64_t>(256, (rows + 128) / 256 * 256);
    c.rec_rows = std::min<int64_t>(rows, (n + 255) / 256 * 256);
    c.rec_rows = std::max<int64_t>(c.rec_rows, c.min_rows);
    c.min_bytes = c.off_z + round_up(size_t(c.min_rows) * c.ldz * 4, kAlign);
    c.rec_bytes = c.off_z + round_up(size_t(c.rec_rows) * c.ldz * 4, kAlign);
    return c;
}

// Workspace of the streaming factor: two device chunk buffers (chunk_rows x B, dense) followed by the
// factor scratch of one chunk.
struct StreamCarve { size_t buf_bytes, bytes; };
StreamCarve stream_carve(int64_t chunk_rows, int64_t d, int64_t B)
{
    StreamCarve sc;
    sc.buf_bytes = round_up(size_t(chunk_rows) * size_t(B) * 4, kAlign);
    sc.bytes = 2 * sc.buf_bytes + carve(chunk_rows, d, B).rec_bytes;
    return sc;
}

// ---------------------------------------------------------------- GEMM launch

enum TileId { TILE_AUTO = 0, TILE_128x128 = 1, TILE_256x128 = 2, TILE_256x256 = 3, TILE_64x128 = 4 };

// Tuning knobs of lpd_set_option.  Atomic, so that setting one while other threads are inside the library is
// well defined: every launch reads the value once.
std::atomic<int> g_pipe_option{2};            // LPD_OPT_GEMM_PIPELINE
std::atomic<int> g_tile_option{TILE_AUTO};   // LPD_OPT_GEMM_TILE
std::atomic<int> g_csr_route{0};              // LPD_OPT_CSR_ROUTE: 0 by density, 1 dense panel, 2 gather
std::atomic<int> g_sweep_grid{0};             // LPD_OPT_SWEEP_GRID: 0 = by row length, else the number of workgroups of a full sweep
std::atomic<int> g_small_path{1};             // LPD_OPT_SMALL_PATH: 1 = one-launch factor for B <= 256, 0 = panel schedule
std::atomic<int> g_fused_scores{1};           // LPD_OPT_FUSED_SCORES: 1 = prediction with up to GEMM_DOT_MAX weight vectors contracts the kernel block in its launch

// Estimated duration of a launch with BM x BN tiles, in units of (CUs x tile elements): a CU holds `per_cu`
// workgroups (registers and LDS: 5 of the 64x128 tile, 3 of the 128x128 tile, 2 of the 256x128 tile of the plain
// product, else 1; fewer where the write-out holds the scores as well), a launch runs in rounds of 256 x per_cu tiles, and a last round that leaves CUs with fewer
// workgroups than they can hold goes faster, though not in proportion (a lone 4-wavefront workgroup cannot keep a
// CU's MFMA pipes full).  `speed` is the measured main-loop rate relative to the 128x128 tile (larger tiles
// move less through LDS and L2 per FLOP).
double launch_cost(const GemmArgs &a, int bm, int bn, int per_cu, double speed)
{
    const int64_t tiles = int64_t((a.M + bm - 1) / bm) * ((a.n_store + bn - 1) / bn);
    const int64_t slots = int64_t(256) * per_cu;
    const int64_t rem = tiles % slots;
    double rounds = double(tiles / slots);
    if (rem > 0) {
        const int64_t deep = (rem + 255) / 256;          // workgroups on the fullest CU in the last round
        rounds += deep >= per_cu ? 1.0 : 0.2 + 0.8 * double(deep) / per_cu;
    }
    return rounds * double(slots) * bm * bn / speed;
}

// Main-loop-plus-write-out rate of a tile relative to the 128x128 tile, measured on launches that fill the chip
// evenly.  The plain product: larger tiles move less through LDS and L2 per FLOP.  The kernel block: the same for
// long contractions; for short ones the write-out of Z weighs as much as the MFMAs, and small tiles, of which a
// CU holds five, overlap the two better than one large workgroup that does one after the other.
double tile_speed(int tile, int epi, int K)
{
    if (epi == EPI_STORE)       // (the small tile re-reads its operands most: worse where W streams from HBM, K beyond 4,096)
        return tile == TILE_256x256 ? 1.04 : tile == TILE_256x128 ? 1.03 : tile == TILE_64x128 ? (K > 4096 ? 0.88 : 0.95) : 1.0;
    // (contracted at once with weight vectors: the write-out's cross-lane sums cost the same per tile whatever its
    // size, so the large tile keeps its edge at any K)
    if (epi == EPI_GAUSS_DOT) return tile == TILE_256x256 ? 1.07 : tile == TILE_64x128 ? 0.9 : 1.0;
    switch (tile) {
    case TILE_256x256: return K >= 512 ? 1.07 : K >= 256 ? 1.04 : K >= 128 ? 1.02 : K >= 64 ? 0.95 : 0.85;
    case TILE_256x128: return K >= 128 ? 1.03 : 0.95;
    case TILE_64x128: return K >= 1024 ? 0.96 : K >= 256 ? 0.975 : K >= 128 ? 1.0 : K >= 64 ? 1.1 : 1.25;
    default: return 1.0;
    }
}

int tile_choice(const GemmArgs &a, int epi)
{
    const int forced = g_tile_option.load(std::memory_order_relaxed);
    if (forced != TILE_AUTO) return forced;
    // What decides, besides the tiles' own rates, is how evenly the tile count fills the chip.  The smallest
    // tile is for launches of few rows (a ragged last panel, a small batch to predict), which the others would
    // spread over a fraction of the CUs, and for kernel blocks over very few features.
    const bool gauss = epi != EPI_STORE;
    const double cost[5] = {0.0,
                            launch_cost(a, 128, 128, epi == EPI_GAUSS_DOT ? 2 : 3, tile_speed(TILE_128x128, epi, a.K)),
                            launch_cost(a, 256, 128, gauss ? 1 : 2, tile_speed(TILE_256x128, epi, a.K)),
                            launch_cost(a, 256, 256, 1, tile_speed(TILE_256x256, epi, a.K)),
                            launch_cost(a, 64, 128, epi == EPI_GAUSS_DOT ? (a.nv > GEMM_DOT_MAX / 2 ? 2 : 3) : gauss ? 5 : 4, tile_speed(TILE_64x128, epi, a.K))};
    int best = TILE_128x128;
    for (int t : {TILE_256x128, TILE_256x256, TILE_64x128})
        if (cost[t] < cost[best] && !(t == TILE_256x128 && epi == EPI_GAUSS_DOT)) best = t;    // (not built for that write-out)
    return best;
}

template <int BM, int BN, int WGM, int WGN, bool ALIGNED, int EPI, int PIPE>
hipError_t launch_one(GemmArgs a, hipStream_t s)
{
    constexpr size_t lds = gemm_lds_bytes<BM, BN, EPI>();
    auto kern = gemm_nt_kernel<BM, BN, WGM, WGN, ALIGNED, EPI, PIPE>;
    // once per instantiation (initialisation of a function-local static is thread-safe): these kernels use
    // more dynamic LDS than the default limit
    static const hipError_t configured = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (configured != hipSuccess) return configured;
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (a.n_store + BN - 1) / BN;
    const int64_t wgs = int64_t(a.tiles_m) * a.tiles_n;
    if (wgs <= 0) return hipSuccess;
    if (wgs > 0x7fffffff) return hipErrorInvalidValue;
    // (up to 32 weight vectors ask for half the slots: the smaller tiles then fit one more workgroup to a CU)
    const size_t lds_launch = EPI == EPI_GAUSS_DOT && a.nv <= GEMM_DOT_MAX / 2 ? gemm_lds_bytes<BM, BN, EPI>(GEMM_DOT_MAX / 2) : lds;
    hipLaunchKernelGGL(kern, dim3(unsigned(wgs)), dim3(WGM * WGN * 64), lds_launch, s, a);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_tile(const GemmArgs &a, bool aligned, int epi, hipStream_t s)
{
    // The pipelined schedule needs the aligned fast path and per-lane byte offsets inside one
    // tile strip that fit 32 bits.
    const int opt = g_pipe_option.load(std::memory_order_relaxed);
    const bool pipe = opt != 0 && aligned && int64_t(BM) * a.lda * 4 < (int64_t(1) << 31) &&
                      int64_t(BN) * a.ldb * 4 < (int64_t(1) << 31);
    if (epi == EPI_GAUSS_DOT) {
        if constexpr (!(BM == 256 && BN == 128)) {
            if (pipe) return launch_one<BM, BN, WGM, WGN, true, EPI_GAUSS_DOT, 1>(a, s);
            return aligned ? launch_one<BM, BN, WGM, WGN, true, EPI_GAUSS_DOT, 0>(a, s)
                           : launch_one<BM, BN, WGM, WGN, false, EPI_GAUSS_DOT, 0>(a, s);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (epi == EPI_GAUSS) {
        // (two staged tiles cost this variant, which also carries the origin, wavefronts per SIMD or spills)
        if (pipe) return launch_one<BM, BN, WGM, WGN, true, EPI_GAUSS, 1>(a, s);
        return aligned ? launch_one<BM, BN, WGM, WGN, true, EPI_GAUSS, 0>(a, s)
                       : launch_one<BM, BN, WGM, WGN, false, EPI_GAUSS, 0>(a, s);
    }
    // two staged tiles: +1.5 % on the 256x256 tile at any K, more on the 128x128 tile at K about 1,000; the
    // 256x128 tile would lose a wavefront per SIMD to the extra registers
    if constexpr (BM == 256 && BN == 256) {
        // the plain product's large tile runs as four wavefronts of 128 x 128 (256 accumulator registers each, one
        // wavefront per SIMD): half the LDS fragment reads per MFMA of the eight-wavefront layout, +1 % at K >= 8,192
        if (pipe && opt == 2) return launch_one<256, 256, 2, 2, true, EPI_STORE, 2>(a, s);
    } else if constexpr (!(BM == 256 && BN == 128)) {
        if (pipe && opt == 2) return launch_one<BM, BN, WGM, WGN, true, EPI_STORE, 2>(a, s);
    }
    if (pipe) return launch_one<BM, BN, WGM, WGN, true, EPI_STORE, 1>(a, s);
    return aligned ? launch_one<BM, BN, WGM, WGN, true, EPI_STORE, 0>(a, s)
                   : launch_one<BM, BN, WGM, WGN, false, EPI_STORE, 0>(a, s);
}

// The narrow tiles (256 x 32 and 256 x 64, four wavefronts down the rows), plain product only.
template <int BN>
hipError_t launch_narrow(const GemmArgs &a, bool aligned, hipStream_t s)
{
    const bool pipe = g_pipe_option.load(std::memory_order_relaxed) != 0 && aligned &&
                      int64_t(256) * a.lda * 4 < (int64_t(1) << 31) && int64_t(BN) * a.ldb * 4 < (int64_t(1) << 31);
    // four staged tiles, requested two at a time: a row's 64 bytes of two consecutive k-tiles are one 128-byte line,
    // and with 196,608 rows in flight on the chip the L2s lose a line between two separate visits (44 GB fetched
    // for 33 GB of G; 33.4 GB and 7 % faster when both halves are requested together)
    if (pipe && g_pipe_option.load(std::memory_order_relaxed) == 2) return launch_one<256, BN, 4, 1, true, EPI_STORE, 4>(a, s);
    if (pipe) return launch_one<256, BN, 4, 1, true, EPI_STORE, 1>(a, s);
    return aligned ? launch_one<256, BN, 4, 1, true, EPI_STORE, 0>(a, s)
                   : launch_one<256, BN, 4, 1, false, EPI_STORE, 0>(a, s);
}

// tiles_n (optional): receives the number of tile columns of the launch (the layout of GemmArgs::P depends on it)
hipError_t launch_gemm(const GemmArgs &a, int epi, hipStream_t s, int *tiles_n = nullptr, bool allow_narrow = true)
{
    const bool aligned = aligned16(a.A) && aligned16(a.B) && a.lda % 4 == 0 && a.ldb % 4 == 0 && a.K % 4 == 0;
    // a plain product with at most 64 columns (a few dozen weight vectors against the rows of G, which it reads
    // once): a narrow tile does a quarter or half of the MFMA work a 128-wide tile would pad it to, and the pass
    // is bound by reading G (33 GB against up to 32 vectors: 6.0 ms instead of 15.9)
    if (epi == EPI_STORE && a.n_store <= 64 && allow_narrow && g_tile_option.load(std::memory_order_relaxed) == TILE_AUTO) {
        if (tiles_n) *tiles_n = 1;
        return a.n_store <= 32 ? launch_narrow<32>(a, aligned, s) : launch_narrow<64>(a, aligned, s);
    }
    int tile = tile_choice(a, epi);
    if (tile == TILE_256x128 && epi == EPI_GAUSS_DOT) tile = TILE_128x128;     // a forced tile this write-out is not built for
    if (tiles_n) *tiles_n = (a.n_store + (tile == TILE_256x256 ? 256 : 128) - 1) / (tile == TILE_256x256 ? 256 : 128);
    switch (tile) {
    case TILE_256x256: return launch_tile<256, 256, 4, 2>(a, aligned, epi, s);
    case TILE_256x128: return launch_tile<256, 128, 4, 2>(a, aligned, epi, s);
    case TILE_64x128: return launch_tile<64, 128, 2, 2>(a, aligned, epi, s);
    default: return launch_tile<128, 128, 2, 2>(a, aligned, epi, s);
    }
}

// F[row, q] = sum over the tile columns of P[t][row][q], in tile order
__global__ __launch_bounds__(256) void dot_reduce_kernel(const float *__restrict__ P, int tiles_n, int64_t rows, int nv,
                                                         float *__restrict__ F, int64_t ldf)
{
    const int64_t total = rows * nv;
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        float s = 0.0f;
        for (int t = 0; t < tiles_n; ++t) s += P[int64_t(t) * total + e];
        const int64_t row = e / nv;
        F[row * ldf + (e - row * nv)] = s;
    }
}

hipError_t launch_dot_reduce(const float *P, int tiles_n, int64_t rows, int nv, float *F, int64_t ldf, hipStream_t s)
{
    const int64_t total = rows * nv;
    if (total <= 0) return hipSuccess;
    const unsigned grid = unsigned(std::min<int64_t>((total + 255) / 256, 4096));
    hipLaunchKernelGGL(dot_reduce_kernel, dim3(grid), dim3(256), 0, s, P, tiles_n, rows, nv, F, ldf);
    return hipGetLastError();
}

// ---------------------------------------------------------------- row kernels

inline unsigned row_grid(int64_t rows, int groups, int64_t cap = 4096)
{
    const int64_t need = (rows + groups - 1) / groups;
    return unsigned(std::max<int64_t>(1, std::min<int64_t>(need, cap)));
}

// out[i] = ||X_i - cen||^2 (cen = nullptr: ||X_i||^2)
hipError_t launch_sqnorm(const float *X, int64_t n, int64_t d, int64_t ldx, const float *cen, float *out, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const bool vec = aligned16(X) && ldx % 4 == 0;
    if (d >= 256) {
        if (vec) hipLaunchKernelGGL((sqnorm_kernel<64, true>), dim3(row_grid(n, 4)), dim3(256), 0, s, X, n, int(d), ldx, cen, out);
        else hipLaunchKernelGGL((sqnorm_kernel<64, false>), dim3(row_grid(n, 4)), dim3(256), 0, s, X, n, int(d), ldx, cen, out);
    } else {
        if (vec) hipLaunchKernelGGL((sqnorm_kernel<8, true>), dim3(row_grid(n, 32)), dim3(256), 0, s, X, n, int(d), ldx, cen, out);
        else hipLaunchKernelGGL((sqnorm_kernel<8, false>), dim3(row_grid(n, 32)), dim3(256), 0, s, X, n, int(d), ldx, cen, out);
    }
    return hipGetLastError();
}

// The origin of the kernel block and the squared norms of X and L relative to it (see centre_kernel):
// the mean of up to 256 landmark rows spread evenly over L.
hipError_t launch_centred_norms(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B,
                                int64_t ldl, float *cen, float *nx, float *nl, hipStream_t s)
{
    if (d > 0 && B > 0) {
        const int rows = int(std::min<int64_t>(B, 256));
        hipLaunchKernelGGL(centre_kernel, dim3(unsigned((d + 63) / 64)), dim3(256), 0, s, L, ldl, int(d), rows,
                           B / rows, cen);
        const hipError_t ec = hipGetLastError();
        if (ec != hipSuccess) return ec;
    }
    hipError_t e = launch_sqnorm(X, n, d, ldx, cen, nx, s);
    if (e != hipSuccess) return e;
    return launch_sqnorm(L, B, d, ldl, cen, nl, s);
}

// n_rows_G: rows of G, the bound a row list is checked against on the device (INDEXED only)
template <int LPR, bool INDEXED, int ROWS>
hipError_t launch_margins_lpr(const float *G, int64_t n_out, int r, int64_t ldg, const int64_t *rows, int64_t n_rows_G,
                              const float *w, float *m, int64_t ms, bool vec, hipStream_t s)
{
    // A full sweep over long rows runs fastest with few rows open at once (about 128 MB of them): 512 workgroups
    // at 32 KB per row, one per CU at 64 KB.  Measured at 16,384 columns: 6.7 TB/s with 4,096 workgroups, 7.2 TB/s
    // with 256.  Shorter rows and row lists (scattered rows) keep a large grid; for a sweep that lasts only tens of
    // microseconds (100,000 rows of 4 KB) one pass of 12,500 workgroups is 3 us faster than 4,096 taking three turns.
    const int forced = g_sweep_grid.load(std::memory_order_relaxed);
    const int64_t cap = (forced > 0 && !INDEXED) ? forced
                        : INDEXED ? 4096 : r < 8192 ? 16384 : std::max<int64_t>(256, (int64_t(4) << 20) / r);
    const unsigned grid = row_grid(n_out, 256 / LPR * ROWS, cap);
    if (vec) hipLaunchKernelGGL((margins_kernel<LPR, true, INDEXED, ROWS>), dim3(grid), dim3(256), 0, s, G, n_out, r, ldg, rows, n_rows_G, w, m, ms);
    else hipLaunchKernelGGL((margins_kernel<LPR, false, INDEXED, ROWS>), dim3(grid), dim3(256), 0, s, G, n_out, r, ldg, rows, n_rows_G, w, m, ms);
    return hipGetLastError();
}

template <bool INDEXED>
hipError_t launch_margins(const float *G, int64_t n_out, int64_t r, int64_t ldg, const int64_t *rows, int64_t n_rows_G,
                          const float *w, float *m, hipStream_t s, int64_t ms = 1)
{
    const bool vec = aligned16(G) && aligned16(w) && ldg % 4 == 0;
    const int ri = int(r);
    if (r >= 1024) return launch_margins_lpr<64, INDEXED, 2>(G, n_out, ri, ldg, rows, n_rows_G, w, m, ms, vec, s);
    if (r >= 256) return launch_margins_lpr<64, INDEXED, 1>(G, n_out, ri, ldg, rows, n_rows_G, w, m, ms, vec, s);
    if (r >= 128) return launch_margins_lpr<32, INDEXED, 1>(G, n_out, ri, ldg, rows, n_rows_G, w, m, ms, vec, s);
    if (r >= 64) return launch_margins_lpr<16, INDEXED, 1>(G, n_out, ri, ldg, rows, n_rows_G, w, m, ms, vec, s);
    return launch_margins_lpr<8, INDEXED, 1>(G, n_out, ri, ldg, rows, n_rows_G, w, m, ms, vec, s);
}

// Up to 8 weight vectors in one pass over the rows (margins_multi_kernel); four rows per wavefront share
// the weight loads for K >= 3, two below.
hipError_t launch_margins_multi(const float *G, int64_t n, int64_t r, int64_t ldg, const float *Ws, int64_t k,
                                int64_t ldws, float *M, int64_t ldm, hipStream_t s)
{
    const bool vec = aligned16(G) && aligned16(Ws) && ldg % 4 == 0 && ldws % 4 == 0;
#define LPD_MM(KK, RR)                                                                                           \
    case KK: {                                                                                                   \
        const unsigned grid = row_grid(n, 4 * RR);                                                               \
        if (vec) hipLaunchKernelGGL((margins_multi_kernel<KK, true, RR>), dim3(grid), dim3(256), 0, s, G, n, int(r), ldg, Ws, ldws, M, ldm); \
        else hipLaunchKernelGGL((margins_multi_kernel<KK, false, RR>), dim3(grid), dim3(256), 0, s, G, n, int(r), ldg, Ws, ldws, M, ldm);    \
    } break
    switch (int(k)) {
        LPD_MM(1, 2); LPD_MM(2, 2); LPD_MM(3, 4); LPD_MM(4, 4); LPD_MM(5, 4); LPD_MM(6, 4); LPD_MM(7, 4); LPD_MM(8, 4);
    }
#undef LPD_MM
    return hipGetLastError();
}

// ---------------------------------------------------------------- factor schedule

struct EventLog {
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;
    bool on = false;
    hipError_t begin(int kind, hipStream_t s)
    {
        if (!on) return hipSuccess;
        Span sp{kind, nullptr, nullptr};
        hipError_t e = hipEventCreate(&sp.a);
        if (e != hipSuccess) return e;
        e = hipEventCreate(&sp.b);
        if (e != hipSuccess) { (void)hipEventDestroy(sp.a); return e; }
        spans.push_back(sp);
        return hipEventRecord(sp.a, s);
    }
    hipError_t end(hipStream_t s) { return on ? hipEventRecord(spans.back().b, s) : hipSuccess; }
    void destroy()
    {
        for (auto &sp : spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
        spans.clear();
    }
};

int check_factor_args(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                      const float *W, int64_t r, int64_t ldw, const float *G, int64_t ldg)
{
    if (n < 0 || d < 0 || B < 0 || r < 0 || r > B || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0 || B == 0) return LPD_OK;
    if (!G) return LPD_ERR_NULL;
    if (ldg < B) return LPD_ERR_LD;
    if (d > 0 && (!X || !L)) return LPD_ERR_NULL;
    if (d > 0 && (ldx < d || ldl < d)) return LPD_ERR_LD;
    if (r > 0 && !W) return LPD_ERR_NULL;
    if (r > 0 && ldw < B) return LPD_ERR_LD;
    return LPD_OK;
}

#define LPD_HIP(call)                                  \
    do {                                               \
        hipError_t e__ = (call);                       \
        if (e__ != hipSuccess) { status = LPD_ERR_HIP; goto done; } \
    } while (0)

// Device address of `scratch` on the current device, looked up once per device and kept.  Two threads that
// meet here for the first time both look it up and store the same value.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_addr[kMaxDevices];

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LPD_ERR_HIP;
    void *ptr = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LPD_ERR_HIP;
        g_scratch_addr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return LPD_OK;
}

// Prediction with the contracted write-out switched off, or with more classifiers than it takes: how a stored
// panel of the kernel block meets the classifiers' weights.  An MFMA product costs the same whatever their number,
// provided the panel has rows for enough workgroups, which it has with few landmarks (rows = 32 Mi / B): from
// kNarrowRows on for the narrow tiles (256 rows each), from kLongPanelRows on for 128-wide tiles of 64 rows.
// Short panels and few classifiers are served by bandwidth-bound sweeps.
constexpr int64_t kSweepClassifiers = 32;   // up to here a short stored panel is consumed by sweeps, above by MFMA
constexpr int64_t kNarrowRows = 32768;
constexpr int64_t kLongPanelRows = 16384;

// What follows a panel of the kernel block: Z (rows x B) times W^T into `out` (factor: out_cols = B, zero fill
// past r; prediction: out_cols = r classifiers, by sweeps of 8 while they are few, else by the MFMA product).
hipError_t consume_panel(const float *Z, int64_t rows, int64_t ldz, int64_t B, const float *W, int64_t r, int64_t ldw,
                         float *out, int64_t ldo, int64_t out_cols, hipStream_t s)
{
    // (16-byte loads for the MFMA tiles' fast path)
    const bool fast = aligned16(Z) && aligned16(W) && ldz % 4 == 0 && ldw % 4 == 0 && B % 4 == 0;
    const bool narrow_pays = fast && rows >= kNarrowRows;
    const bool mfma_pays = fast && rows >= kLongPanelRows;
    if (out_cols != B && (r <= 4 || (r <= 8 && !narrow_pays) || (r <= kSweepClassifiers && !mfma_pays))) {
        // a few classifiers: bandwidth-bound passes over the panel, 8 classifiers each, instead of an
        // MFMA tile that would be three quarters padding or more; from five classifiers on a narrow MFMA tile
        // reads the panel faster, provided the panel has rows for enough such tiles (few landmarks)
        for (int64_t q0 = 0; q0 < r; q0 += 8) {
            const hipError_t e = launch_margins_multi(Z, rows, B, ldz, W + q0 * ldw, std::min<int64_t>(8, r - q0), ldw,
                                                      out + q0, ldo, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    GemmArgs k2{};
    k2.A = Z; k2.lda = ldz;
    k2.B = W; k2.ldb = ldw;
    k2.C = out; k2.ldc = ldo;
    k2.M = int(rows); k2.N = int(r); k2.K = int(B); k2.n_store = int(out_cols);
    // (33 to 64 classifiers against a short panel: a 128-wide tile of 64 rows, half of it padding, still spreads
    // over four times as many workgroups as the narrow tile)
    return launch_gemm(k2, EPI_STORE, s, nullptr, out_cols == B || narrow_pays);
}

// Shared schedule of the factor (out_cols = B: G = Z W^T with zero fill of columns r..B-1) and of
// prediction (out_cols = r = number of classifiers, W = their folded weight rows: F = Z V^T).
int factor_impl(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                float gamma, const float *W, int64_t r, int64_t ldw, float *G, int64_t ldg, int64_t out_cols,
                void *workspace, size_t workspace_bytes, hipStream_t s, lpd_factor_profile *prof)
{
    int status = check_factor_args(X, n, d, ldx, L, B, ldl, W, r, ldw, G, out_cols == B ? ldg : std::max(ldg, B));
    if (status == LPD_OK && ldg < out_cols) status = LPD_ERR_LD;
    if (prof) std::memset(prof, 0, sizeof(*prof));
    if (status != LPD_OK || n == 0 || B == 0) return status;

    const Carve c = carve(n, d, B);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < c.min_bytes)
        return LPD_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    float *nx = reinterpret_cast<float *>(ws + c.off_nx);
    float *nl = reinterpret_cast<float *>(ws + c.off_nl);
    float *cen = reinterpret_cast<float *>(ws + c.off_cen);
    float *Z = reinterpret_cast<float *>(ws + c.off_z);
    int64_t panel = int64_t((workspace_bytes - c.off_z) / (size_t(c.ldz) * 4));
    if (panel >= n) panel = n;
    else panel = std::max<int64_t>(c.min_rows, panel / 256 * 256);

    EventLog log;
    log.on = prof != nullptr;
    bool fused_scores = false;

    // Few landmarks: the whole of step 1d in one launch (fused_small.hip.h); the workspace is not touched.
    if (out_cols == B && B <= SM_MAXB && d <= SM_MAXD && g_small_path.load(std::memory_order_relaxed) != 0) {
        SmallArgs a{};
        a.X = X; a.L = L; a.W = W; a.G = G;
        a.ldx = ldx; a.ldl = ldl; a.ldw = ldw; a.ldg = ldg;
        a.n = int(n); a.d = int(d); a.B = int(B); a.r = int(r);
        a.cen_rows = int(std::min<int64_t>(B, 32));
        a.cen_step = int(B / a.cen_rows);
        a.scale = -gamma * 1.44269504088896340736f;
        const bool vec = d % 4 == 0 && B % 4 == 0 && ldx % 4 == 0 && ldl % 4 == 0 && aligned16(X) && aligned16(L) &&
                         (r == 0 || (ldw % 4 == 0 && aligned16(W)));
        const dim3 grid(unsigned((n + SM_TM - 1) / SM_TM));
        LPD_HIP(log.begin(2, s));
        if (vec) hipLaunchKernelGGL((nystrom_small_kernel<true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((nystrom_small_kernel<false>), grid, dim3(256), 0, s, a);
        LPD_HIP(hipGetLastError());
        LPD_HIP(log.end(s));
        panel = n;
        goto readout;
    }

    LPD_HIP(log.begin(0, s));
    LPD_HIP(launch_centred_norms(X, n, d, ldx, L, B, ldl, cen, nx, nl, s));
    LPD_HIP(log.end(s));

    // (the shares of the scores, one per 128 landmarks at most, must fit a panel row's place in the workspace)
    fused_scores = out_cols != B && r > 0 && r <= GEMM_DOT_MAX && g_fused_scores.load(std::memory_order_relaxed) != 0 &&
                   ((B + 127) / 128) * r <= c.ldz;
    if (fused_scores && panel < n) {
        // no panel of the kernel block is stored, so a launch can take as many rows as their shares of the scores
        // fit the workspace: fewer launches, fewer ragged ends
        int64_t fit = int64_t((workspace_bytes - c.off_z) / 4) / (((B + 127) / 128) * r) / 256 * 256;
        // (whole rounds of 256x256 tiles over the 256 CUs where the rows allow: tile rows x tile columns a multiple of 256)
        const int64_t even = 256 * (256 / std::gcd<int64_t>(256, (B + 255) / 256));
        if (fit >= even) fit = fit / even * even;
        panel = std::min<int64_t>(n, std::max<int64_t>(panel, fit));
    }
    for (int64_t p0 = 0; p0 < n; p0 += panel) {
        const int64_t rows = std::min<int64_t>(panel, n - p0);
        GemmArgs k1{};
        k1.A = X + p0 * ldx; k1.lda = ldx;
        k1.B = L; k1.ldb = ldl;
        k1.C = Z; k1.ldc = c.ldz;
        k1.M = int(rows); k1.N = int(B); k1.K = int(d); k1.n_store = int(B);
        k1.na = nx + p0; k1.nb = nl; k1.cen = cen;
        k1.scale = -gamma * 1.44269504088896340736f;
        if (fused_scores) {
            // prediction with few weight vectors: the kernel block is contracted with them in the write-out of
            // the same launch and never written; the panel's place in the workspace takes the per-tile-column
            // shares of the scores, which one small pass adds up
            k1.C = nullptr;
            k1.V = W; k1.ldv = ldw; k1.nv = int(r); k1.P = Z;
            int tiles_n = 0;
            LPD_HIP(log.begin(1, s));
            LPD_HIP(launch_gemm(k1, EPI_GAUSS_DOT, s, &tiles_n));
            LPD_HIP(log.end(s));
            LPD_HIP(log.begin(2, s));
            LPD_HIP(launch_dot_reduce(Z, tiles_n, rows, int(r), G + p0 * ldg, ldg, s));
            LPD_HIP(log.end(s));
            continue;
        }
        LPD_HIP(log.begin(1, s));
        LPD_HIP(launch_gemm(k1, EPI_GAUSS, s));
        LPD_HIP(log.end(s));

        LPD_HIP(log.begin(2, s));
        LPD_HIP(consume_panel(Z, rows, c.ldz, B, W, r, ldw, G + p0 * ldg, ldg, out_cols, s));
        LPD_HIP(log.end(s));
    }

readout:
    if (prof) {
        LPD_HIP(hipStreamSynchronize(s));
        prof->panel_rows = int32_t(panel);
        for (auto &sp : log.spans) {
            float ms = 0.f;
            LPD_HIP(hipEventElapsedTime(&ms, sp.a, sp.b));
            if (sp.kind == 0) { prof->ms_norms += ms; prof->launches_norms += 3; }
            else if (sp.kind == 1) { prof->ms_kernel_block += ms; prof->launches_kernel_block += 1; }
            else { prof->ms_whiten += ms; prof->launches_whiten += 1; }
        }
    }
done:
    log.destroy();
    return status;
}

// The compressed-row entry points take one of two routes.  Dense-panel route: each chunk of rows is written
// out into a dense panel and handed to the dense MFMA schedule.  Gather route, for rows so sparse that the
// written-out zeros would dominate: the kernel block is accumulated entry by entry from the transposed
// landmarks.  The switch is the density nnz / (n d) against kGatherDensity; an unknown nnz (< 0) takes the
// dense-panel route.  Measured on 1,000,000 x 784 rows against 4,096 landmarks, kernel-block share of the
// factor: dense panels 45 ms at any density; gather 2 / 4 / 7.5 / 12 / 21 / 43 ms at 0.5 / 1 / 2 / 3 / 5 / 10 %
// non-zeros.  Both scale with n d B, so the break-even near 10 % carries over to other shapes.
constexpr double kGatherDensity = 0.08;

bool csr_use_gather(int64_t n, int64_t d, int64_t nnz)
{
    const int route = g_csr_route.load(std::memory_order_relaxed);
    if (route != 0) return route == 2;
    return nnz >= 0 && n > 0 && d > 0 && double(nnz) < kGatherDensity * double(n) * double(d);
}

// Workspace.  Dense-panel route: the panel (chunk_rows x ldxd, ldxd = d rounded up to 4) and the dense
// call's scratch.  Gather route: the transposed landmarks (d x ldlt, ldlt = B rounded up to 4), the
// landmark norms, and a panel of the kernel block (chunk_rows x ldz) for the product that follows.
struct CsrCarve { bool gather; int64_t ldxd, ldlt, ldz; size_t panel_bytes, off_nl, off_z, bytes; };
CsrCarve csr_carve(int64_t chunk_rows, int64_t d, int64_t B, bool gather)
{
    CsrCarve c{};
    c.gather = gather;
    c.ldxd = std::max<int64_t>(4, (d + 3) / 4 * 4);
    c.ldlt = std::max<int64_t>(4, (B + 3) / 4 * 4);
    c.ldz = panel_ld(B);
    if (gather) {
        c.panel_bytes = round_up(size_t(std::max<int64_t>(d, 1)) * size_t(c.ldlt) * 4, kAlign);     // Lt
        c.off_nl = c.panel_bytes;
        c.off_z = c.off_nl + round_up(size_t(B) * 4, kAlign);
        c.bytes = c.off_z + round_up(size_t(chunk_rows) * size_t(c.ldz) * 4, kAlign);
    } else {
        c.panel_bytes = round_up(size_t(chunk_rows) * size_t(c.ldxd) * 4, kAlign);
        c.bytes = c.panel_bytes + carve(chunk_rows, d, B).rec_bytes;
    }
    return c;
}

int lpd_kernel_block_dense(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                           float gamma, float *Z, int64_t ldz, void *workspace, size_t workspace_bytes, hipStream_t s)
{
    if (n < 0 || d < 0 || B < 0 || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0 || B == 0) return LPD_OK;
    if (!Z) return LPD_ERR_NULL;
    if (ldz < B) return LPD_ERR_LD;
    if (d > 0 && (!X || !L)) return LPD_ERR_NULL;
    if (d > 0 && (ldx < d || ldl < d)) return LPD_ERR_LD;
    const Carve c = carve(n, d, B);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < c.off_z)
        return LPD_ERR_WORKSPACE;
    float *nx = reinterpret_cast<float *>(workspace);
    float *nl = reinterpret_cast<float *>(static_cast<char *>(workspace) + c.off_nl);
    float *cen = reinterpret_cast<float *>(static_cast<char *>(workspace) + c.off_cen);
    if (launch_centred_norms(X, n, d, ldx, L, B, ldl, cen, nx, nl, s) != hipSuccess) return LPD_ERR_HIP;
    GemmArgs k1{};
    k1.A = X; k1.lda = ldx;
    k1.B = L; k1.ldb = ldl;
    k1.C = Z; k1.ldc = ldz;
    k1.M = int(n); k1.N = int(B); k1.K = int(d); k1.n_store = int(B);
    k1.na = nx; k1.nb = nl; k1.cen = cen;
    k1.scale = -gamma * 1.44269504088896340736f;
    return launch_gemm(k1, EPI_GAUSS, s) == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

// factor: G = K(X, L) W^T; prediction: F = K(X, L) V^T; otherwise Z = K(X, L), for X in compressed-row form.
int csr_impl(const int64_t *row_ptr, const int32_t *col_idx, const float *values, int64_t n, int64_t d, int64_t nnz,
             const float *L, int64_t B, int64_t ldl, float gamma, const float *W, int64_t r, int64_t ldw, float *out,
             int64_t ldo, int64_t chunk_rows, void *workspace, size_t workspace_bytes, hipStream_t s, int mode)
{
    // mode 0: Z = K(X, L);  1: G = K(X, L) W^T (n x B, zero-filled past r);  2: F = K(X, L) V^T (n x r scores)
    const bool factor = mode != 0;
    const int64_t out_cols = mode == 2 ? r : B;
    if (n < 0 || d < 0 || B < 0 || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    if (factor && (r < 0 || r > B)) return LPD_ERR_SHAPE;
    if (n == 0 || B == 0) return LPD_OK;
    if (chunk_rows <= 0 || chunk_rows > kMaxDim) return LPD_ERR_SHAPE;
    if (!row_ptr || !out || (d > 0 && !L) || (factor && r > 0 && !W)) return LPD_ERR_NULL;
    if (ldo < out_cols || (d > 0 && ldl < d) || (factor && ldw < B)) return LPD_ERR_LD;
    if (mode == 2 && r == 0) return LPD_OK;
    chunk_rows = std::min(chunk_rows, n);
    const CsrCarve cc = csr_carve(chunk_rows, d, B, csr_use_gather(n, d, nnz));
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < cc.bytes)
        return LPD_ERR_WORKSPACE;
    char *wsp = static_cast<char *>(workspace);

    if (cc.gather) {
        float *Lt = reinterpret_cast<float *>(wsp);
        float *nl = reinterpret_cast<float *>(wsp + cc.off_nl);
        float *Zp = reinterpret_cast<float *>(wsp + cc.off_z);
        hipLaunchKernelGGL(transpose_kernel, dim3(unsigned((B + 31) / 32), unsigned((d + 31) / 32)), dim3(256), 0, s, L,
                           int(B), int(d), ldl, Lt, cc.ldlt);
        if (hipGetLastError() != hipSuccess || launch_sqnorm(L, B, d, ldl, nullptr, nl, s) != hipSuccess) return LPD_ERR_HIP;
        const float scale = -gamma * 1.44269504088896340736f;
        for (int64_t c0 = 0; c0 < n; c0 += chunk_rows) {
            const int64_t rows = std::min(chunk_rows, n - c0);
            float *Zout = factor ? Zp : out + c0 * ldo;
            const int64_t ldzo = factor ? cc.ldz : ldo;
            const dim3 grid(unsigned((B + 1023) / 1024), unsigned(std::min<int64_t>(rows, 16384)));
            hipLaunchKernelGGL(csr_gauss_gather_kernel, grid, dim3(256), 0, s, row_ptr, col_idx, values, c0, rows, int(d),
                               Lt, int(B), cc.ldlt, nl, scale, Zout, ldzo);
            if (hipGetLastError() != hipSuccess) return LPD_ERR_HIP;
            if (factor && consume_panel(Zp, rows, cc.ldz, B, W, r, ldw, out + c0 * ldo, ldo, out_cols, s) != hipSuccess)
                return LPD_ERR_HIP;
        }
        return LPD_OK;
    }

    float *Xd = reinterpret_cast<float *>(wsp);
    void *dws = wsp + cc.panel_bytes;
    const size_t dws_bytes = workspace_bytes - cc.panel_bytes;
    for (int64_t c0 = 0; c0 < n; c0 += chunk_rows) {
        const int64_t rows = std::min(chunk_rows, n - c0);
        const int64_t count4 = rows * cc.ldxd / 4;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(unsigned(std::min<int64_t>(4096, (count4 + 255) / 256))), dim3(256), 0,
                           s, reinterpret_cast<rf32x4 *>(Xd), count4);
        if (col_idx && values)
            hipLaunchKernelGGL(csr_scatter_kernel, dim3(row_grid(rows, 4)), dim3(256), 0, s, row_ptr, col_idx, values,
                               c0, rows, int(d), Xd, cc.ldxd);
        if (hipGetLastError() != hipSuccess) return LPD_ERR_HIP;
        const int st = factor
            ? factor_impl(Xd, rows, d, cc.ldxd, L, B, ldl, gamma, W, r, ldw, out + c0 * ldo, ldo, out_cols, dws,
                          dws_bytes, s, nullptr)
            : lpd_kernel_block_dense(Xd, rows, d, cc.ldxd, L, B, ldl, gamma, out + c0 * ldo, ldo, dws, dws_bytes, s);
        if (st != LPD_OK) return st;
    }
    return LPD_OK;
}

}  // namespace

extern "C" {

int lpd_version(void) { return 100; }

const char *lpd_strerror(int status)
{
    switch (status) {
    case LPD_OK: return "ok";
    case LPD_ERR_NULL: return "a required pointer is NULL";
    case LPD_ERR_SHAPE: return "invalid size (negative, r > B, or above the supported limit)";
    case LPD_ERR_LD: return "leading dimension smaller than the row length";
    case LPD_ERR_WORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case LPD_ERR_HIP: return "HIP runtime call or kernel launch failed";
    case LPD_ERR_NUMERIC: return "eigendecomposition failed or kernel matrix not positive";
    case LPD_ERR_LIMIT: return "sizes need more than the fixed 32 MiB scratch of the allocation-free entry point";
    default: return "unknown status";
    }
}

int lpd_set_option(int option, int64_t value)
{
    if (option == LPD_OPT_GEMM_TILE && value >= TILE_AUTO && value <= TILE_64x128) {
        g_tile_option.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    if (option == LPD_OPT_CSR_ROUTE && value >= 0 && value <= 2) {
        g_csr_route.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    if (option == LPD_OPT_SWEEP_GRID && value >= 0 && value <= 65536) {
        g_sweep_grid.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    if (option == LPD_OPT_WHITEN_UPPER && (value == 0 || value == 1)) {
        lpd_host::set_upper_triangle_pass(int(value));
        return LPD_OK;
    }
    if (option == LPD_OPT_WHITEN_DC && (value == 0 || value == 1)) {
        lpd_host::set_divide_and_conquer(int(value));
        return LPD_OK;
    }
    if (option == LPD_OPT_FUSED_SCORES && (value == 0 || value == 1)) {
        g_fused_scores.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    if (option == LPD_OPT_SMALL_PATH && (value == 0 || value == 1)) {
        g_small_path.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    if (option == LPD_OPT_GEMM_PIPELINE && value >= 0 && value <= 2) {
        g_pipe_option.store(int(value), std::memory_order_relaxed);
        return LPD_OK;
    }
    return LPD_ERR_SHAPE;
}

int lpd_nystrom_factor_workspace(int64_t n, int64_t d, int64_t B, size_t *bytes, size_t *min_bytes)
{
    if (!bytes) return LPD_ERR_NULL;
    if (n < 0 || d < 0 || B < 0 || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    const Carve c = carve(n, d, B);
    *bytes = c.rec_bytes;
    if (min_bytes) *min_bytes = c.min_bytes;
    return LPD_OK;
}

int lpd_nystrom_factor(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                       float gamma, const float *W, int64_t r, int64_t ldw, float *G, int64_t ldg,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return factor_impl(X, n, d, ldx, L, B, ldl, gamma, W, r, ldw, G, ldg, B, workspace, workspace_bytes,
                       static_cast<hipStream_t>(hip_stream), nullptr);
}

int lpd_nystrom_factor_profiled(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B,
                                int64_t ldl, float gamma, const float *W, int64_t r, int64_t ldw, float *G,
                                int64_t ldg, void *workspace, size_t workspace_bytes, void *hip_stream,
                                lpd_factor_profile *profile)
{
    if (!profile) return LPD_ERR_NULL;
    return factor_impl(X, n, d, ldx, L, B, ldl, gamma, W, r, ldw, G, ldg, B, workspace, workspace_bytes,
                       static_cast<hipStream_t>(hip_stream), profile);
}

int lpd_nystrom_factor_to_host_workspace(int64_t n, int64_t d, int64_t B, int64_t *chunk_rows, size_t *bytes)
{
    if (!chunk_rows || !bytes) return LPD_ERR_NULL;
    if (n < 0 || d < 0 || B < 0 || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    if (*chunk_rows <= 0) *chunk_rows = std::max<int64_t>(1, std::min<int64_t>(n, carve(n, d, B).rec_rows));
    if (*chunk_rows > kMaxDim) return LPD_ERR_SHAPE;
    const StreamCarve sc = stream_carve(*chunk_rows, d, B);
    *bytes = sc.bytes;
    return LPD_OK;
}

int lpd_nystrom_factor_to_host(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B,
                               int64_t ldl, float gamma, const float *W, int64_t r, int64_t ldw, float *G_host,
                               int64_t ldg, int64_t chunk_rows, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    int status = check_factor_args(X, n, d, ldx, L, B, ldl, W, r, ldw, G_host, ldg);
    if (status != LPD_OK) return status;
    if (chunk_rows <= 0 || chunk_rows > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0 || B == 0) return LPD_OK;
    chunk_rows = std::min(chunk_rows, n);
    const StreamCarve sc = stream_carve(chunk_rows, d, B);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < sc.bytes)
        return LPD_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    float *buf[2] = {reinterpret_cast<float *>(ws), reinterpret_cast<float *>(ws + sc.buf_bytes)};
    void *fws = ws + 2 * sc.buf_bytes;
    const size_t fws_bytes = workspace_bytes - 2 * sc.buf_bytes;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipStream_t cs = nullptr;
    hipEvent_t computed[2] = {nullptr, nullptr}, copied[2] = {nullptr, nullptr};
    LPD_HIP(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
    for (int b = 0; b < 2; ++b) {
        LPD_HIP(hipEventCreateWithFlags(&computed[b], hipEventDisableTiming));
        LPD_HIP(hipEventCreateWithFlags(&copied[b], hipEventDisableTiming));
    }
    {
        int64_t chunk = 0;
        for (int64_t c0 = 0; c0 < n; c0 += chunk_rows, ++chunk) {
            const int64_t rows = std::min(chunk_rows, n - c0);
            const int b = int(chunk & 1);
            // the buffer is free again once the copy of the chunk before last has drained
            if (chunk >= 2) LPD_HIP(hipStreamWaitEvent(s, copied[b], 0));
            status = factor_impl(X + c0 * ldx, rows, d, ldx, L, B, ldl, gamma, W, r, ldw, buf[b], B, B, fws,
                                 fws_bytes, s, nullptr);
            if (status != LPD_OK) break;
            LPD_HIP(hipEventRecord(computed[b], s));
            LPD_HIP(hipStreamWaitEvent(cs, computed[b], 0));
            LPD_HIP(hipMemcpy2DAsync(G_host + c0 * ldg, size_t(ldg) * 4, buf[b], size_t(B) * 4, size_t(B) * 4,
                                     size_t(rows), hipMemcpyDeviceToHost, cs));
            LPD_HIP(hipEventRecord(copied[b], cs));
        }
    }
done:
    // drain both streams before the events and the buffers they guard go away, on errors too
    if (cs && hipStreamSynchronize(cs) != hipSuccess && status == LPD_OK) status = LPD_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess && status == LPD_OK) status = LPD_ERR_HIP;
    for (int b = 0; b < 2; ++b) {
        if (computed[b]) (void)hipEventDestroy(computed[b]);
        if (copied[b]) (void)hipEventDestroy(copied[b]);
    }
    if (cs) (void)hipStreamDestroy(cs);
    return status;
}

int lpd_nystrom_factor_csr_workspace(int64_t n, int64_t d, int64_t B, int64_t nnz, int64_t *chunk_rows, size_t *bytes)
{
    if (!chunk_rows || !bytes) return LPD_ERR_NULL;
    if (n < 0 || d < 0 || B < 0 || n > kMaxDim || d > kMaxDim || B > kMaxDim) return LPD_ERR_SHAPE;
    if (*chunk_rows <= 0) *chunk_rows = std::max<int64_t>(1, std::min<int64_t>(n, carve(n, d, B).rec_rows));
    if (*chunk_rows > kMaxDim) return LPD_ERR_SHAPE;
    *bytes = csr_carve(*chunk_rows, d, B, csr_use_gather(n, d, nnz)).bytes;
    return LPD_OK;
}

int lpd_nystrom_factor_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values, int64_t n, int64_t d, int64_t nnz,
                           const float *L, int64_t B, int64_t ldl, float gamma, const float *W, int64_t r, int64_t ldw,
                           float *G, int64_t ldg, int64_t chunk_rows, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    return csr_impl(row_ptr, col_idx, values, n, d, nnz, L, B, ldl, gamma, W, r, ldw, G, ldg, chunk_rows, workspace,
                    workspace_bytes, static_cast<hipStream_t>(hip_stream), 1);
}

int lpd_predict_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values, int64_t n, int64_t d, int64_t nnz,
                    const float *L, int64_t B, int64_t ldl, float gamma, const float *V, int64_t c, int64_t ldv,
                    float *F, int64_t ldf, int64_t chunk_rows, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return csr_impl(row_ptr, col_idx, values, n, d, nnz, L, B, ldl, gamma, V, c, ldv, F, ldf, chunk_rows, workspace,
                    workspace_bytes, static_cast<hipStream_t>(hip_stream), 2);
}

int lpd_kernel_block_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values, int64_t n, int64_t d, int64_t nnz,
                         const float *L, int64_t B, int64_t ldl, float gamma, float *Z, int64_t ldz, int64_t chunk_rows,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return csr_impl(row_ptr, col_idx, values, n, d, nnz, L, B, ldl, gamma, nullptr, 0, B, Z, ldz, chunk_rows, workspace,
                    workspace_bytes, static_cast<hipStream_t>(hip_stream), 0);
}

int lpd_kernel_block(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                     float gamma, float *Z, int64_t ldz, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return lpd_kernel_block_dense(X, n, d, ldx, L, B, ldl, gamma, Z, ldz, workspace, workspace_bytes,
                                  static_cast<hipStream_t>(hip_stream));
}

int lpd_margins(const float *G, int64_t n, int64_t r, int64_t ldg, const float *w, float *m, void *hip_stream)
{
    if (n < 0 || r < 0 || n > kMaxDim * 4 || r > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0) return LPD_OK;
    if (!m) return LPD_ERR_NULL;
    if (r > 0 && (!G || !w)) return LPD_ERR_NULL;
    if (ldg < r) return LPD_ERR_LD;
    hipError_t e = launch_margins<false>(G, n, r, ldg, nullptr, n, w, m, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

int lpd_margins_rows(const float *G, int64_t n, int64_t r, int64_t ldg, const int64_t *rows, int64_t n_rows,
                     const float *w, float *m, void *hip_stream)
{
    if (n < 0 || r < 0 || n_rows < 0 || n > kMaxDim * 4 || r > kMaxDim || n_rows > kMaxDim * 4) return LPD_ERR_SHAPE;
    if (n_rows == 0) return LPD_OK;
    if (n == 0) return LPD_ERR_SHAPE;        // rows listed, but G has none
    if (!m || !rows) return LPD_ERR_NULL;
    if (r > 0 && (!G || !w)) return LPD_ERR_NULL;
    if (ldg < r) return LPD_ERR_LD;
    hipError_t e = launch_margins<true>(G, n_rows, r, ldg, rows, n, w, m, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

int lpd_margins_multi(const float *G, int64_t n, int64_t r, int64_t ldg, const float *Ws, int64_t k, int64_t ldws,
                      float *M, int64_t ldm, void *hip_stream)
{
    if (n < 0 || r < 0 || k < 0 || n > kMaxDim || r > kMaxDim || k > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0 || k == 0) return LPD_OK;
    if (!M || (r > 0 && (!G || !Ws))) return LPD_ERR_NULL;
    if (ldg < r || ldws < r || ldm < k) return LPD_ERR_LD;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // From five vectors on the MFMA product M = G Ws^T on a narrow tile reads G faster than the plain kernel, whose
    // inner products are vector FMAs (6 vectors against 34 GB of G: 6.0 ms instead of 6.3; rows of 256: 28 us instead
    // of 52); operands the tile's 16-byte loader cannot take stay with the plain kernel up to its 8 vectors.
    const bool fast = aligned16(G) && aligned16(Ws) && ldg % 4 == 0 && ldws % 4 == 0 && r % 4 == 0;
    if (k > 8 || (k > 4 && fast)) {
        GemmArgs a{};
        a.A = G; a.lda = ldg;
        a.B = Ws; a.ldb = ldws;
        a.C = M; a.ldc = ldm;
        a.M = int(n); a.N = int(k); a.K = int(r); a.n_store = int(k);
        return launch_gemm(a, EPI_STORE, s) == hipSuccess ? LPD_OK : LPD_ERR_HIP;
    }
    return launch_margins_multi(G, n, r, ldg, Ws, k, ldws, M, ldm, s) == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

int lpd_fold_weights(const float *W, int64_t r, int64_t B, int64_t ldw, const float *Ws, int64_t c, int64_t ldws,
                     float *V, int64_t ldv, void *hip_stream)
{
    if (r < 0 || B < 0 || c < 0 || r > kMaxDim || B > kMaxDim || c > 65535 * 8) return LPD_ERR_SHAPE;
    if (c == 0 || B == 0) return LPD_OK;
    if (!V || (r > 0 && (!W || !Ws))) return LPD_ERR_NULL;
    if (ldv < B || (r > 0 && (ldw < B || ldws < r))) return LPD_ERR_LD;
    constexpr int CPT = 8;
    const dim3 grid(unsigned((B + 255) / 256), unsigned((c + CPT - 1) / CPT));
    hipLaunchKernelGGL((fold_weights_kernel<CPT>), grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream), W,
                       int(r), int(B), ldw, Ws, int(c), ldws, V, ldv);
    return hipGetLastError() == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

int lpd_predict(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                float gamma, const float *V, int64_t c, int64_t ldv, float *F, int64_t ldf, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    if (c < 0 || c > B) return LPD_ERR_SHAPE;
    if (c == 0) return LPD_OK;
    return factor_impl(X, n, d, ldx, L, B, ldl, gamma, V, c, ldv, F, ldf, c == B ? B : c, workspace, workspace_bytes,
                       static_cast<hipStream_t>(hip_stream), nullptr);
}

int lpd_predict_noalloc(const float *X, int64_t n, int64_t d, int64_t ldx, const float *L, int64_t B, int64_t ldl,
                        float gamma, const float *V, int64_t c, int64_t ldv, float *F, int64_t ldf, void *hip_stream)
{
    if (c < 0 || c > B) return LPD_ERR_SHAPE;
    const int64_t out_cols = c == B ? B : c;
    int status = check_factor_args(X, n, d, ldx, L, B, ldl, V, c, ldv, F, std::max(ldf, B));
    if (status == LPD_OK && ldf < out_cols) status = LPD_ERR_LD;
    if (status != LPD_OK || c == 0 || n == 0 || B == 0) return status;
    // the smallest workspace lpd_predict accepts for this shape must fit the fixed array
    if (carve(n, d, B).min_bytes > kStaticScratchBytes) return LPD_ERR_LIMIT;
    void *ws = nullptr;
    status = static_scratch(&ws);
    if (status != LPD_OK) return status;
    return factor_impl(X, n, d, ldx, L, B, ldl, gamma, V, c, ldv, F, ldf, out_cols, ws, kStaticScratchBytes,
                       static_cast<hipStream_t>(hip_stream), nullptr);
}

int lpd_row_sqnorms(const float *G, int64_t n, int64_t r, int64_t ldg, float *gsq, void *hip_stream)
{
    if (n < 0 || r < 0 || n > kMaxDim * 4 || r > kMaxDim) return LPD_ERR_SHAPE;
    if (n == 0) return LPD_OK;
    if (!gsq || (r > 0 && !G)) return LPD_ERR_NULL;
    if (ldg < r) return LPD_ERR_LD;
    return launch_sqnorm(G, n, r, ldg, nullptr, gsq, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

int lpd_cd_solve_workspace(int64_t n_problems, int64_t total_rows, size_t *bytes)
{
    if (!bytes) return LPD_ERR_NULL;
    if (n_problems < 0 || total_rows < 0 || n_problems > kMaxDim || total_rows > kMaxDim) return LPD_ERR_SHAPE;
    *bytes = round_up(size_t(3) * size_t(total_rows + n_problems) * 4, kAlign) + round_up(size_t(total_rows), kAlign);
    return LPD_OK;
}

int lpd_cd_solve(const float *G, int64_t n, int64_t r, int64_t ldg, const float *gsq, int64_t n_problems,
                 const int64_t *prob_off, int64_t total_rows, const int64_t *rows, const float *y, const float *C,
                 float *alpha, float *w, int64_t ldw, lpd_cd_status *status, float eps, int32_t max_epochs,
                 int32_t shrink_k, float eta, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    static_assert(sizeof(lpd_cd_status) == sizeof(CdStatus), "status record layout");
    if (n < 0 || r < 0 || n_problems < 0 || total_rows < 0 || n > kMaxDim || n_problems > 0x7fffffff ||
        total_rows > kMaxDim || r > 16384 || max_epochs < 0 || shrink_k < 0 || shrink_k > 255 ||
        !(eta >= 0.0f && eta < 1.0f) || !(eps >= 0.0f))
        return LPD_ERR_SHAPE;
    if (n_problems == 0) return LPD_OK;
    // rows are read 16 bytes at a time from column 0 on: a factor without columns, or without rows, has
    // nothing to read them from
    if (total_rows > 0 && (r == 0 || n == 0)) return LPD_ERR_SHAPE;
    if (!prob_off || !C || !status || (r > 0 && !w)) return LPD_ERR_NULL;
    if (total_rows > 0 && (!rows || !y || !alpha || !gsq || !G)) return LPD_ERR_NULL;
    if (ldg < r || ldw < r) return LPD_ERR_LD;
    size_t need = 0;
    lpd_cd_solve_workspace(n_problems, total_rows, &need);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < need)
        return LPD_ERR_WORKSPACE;

    CdArgs a{};
    a.G = G; a.ldg = ldg; a.r = int(r); a.n = n; a.gsq = gsq;
    a.prob_off = prob_off; a.rows = rows; a.y = y; a.C = C; a.alpha = alpha;
    a.w = w; a.ldw = ldw; a.status = reinterpret_cast<CdStatus *>(status);
    a.lists = static_cast<int32_t *>(workspace);
    a.cnt = static_cast<uint8_t *>(workspace) + round_up(size_t(3) * size_t(total_rows + n_problems) * 4, kAlign);
    a.total = total_rows; a.n_problems = n_problems;
    a.eps = eps; a.max_epochs = max_epochs; a.shrink_k = shrink_k;
    a.check_every = eta > 0.0f ? int(std::floor((1.0 - double(eta)) / double(eta) + 0.5)) : 0;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const dim3 grid{unsigned(n_problems)};
    const bool vec = ldg % 4 == 0 && aligned16(G);
#define LPD_CD_LAUNCH(WV, NC)                                                                       \
    do {                                                                                            \
        if (vec && r == 256 * WV * NC) hipLaunchKernelGGL((cd_solve_kernel<WV, NC, 2>), grid, dim3(64 * WV), 0, s, a); \
        else if (vec) hipLaunchKernelGGL((cd_solve_kernel<WV, NC, 1>), grid, dim3(64 * WV), 0, s, a); \
        else hipLaunchKernelGGL((cd_solve_kernel<WV, NC, 0>), grid, dim3(64 * WV), 0, s, a);    \
    } while (0)
    if (r <= 256) LPD_CD_LAUNCH(1, 1);
    else if (r <= 512) LPD_CD_LAUNCH(1, 2);
    else if (r <= 1024) LPD_CD_LAUNCH(1, 4);
    else if (r <= 2048) LPD_CD_LAUNCH(1, 8);
    else if (r <= 4096) LPD_CD_LAUNCH(1, 16);
    else if (r <= 8192) LPD_CD_LAUNCH(4, 8);
    else LPD_CD_LAUNCH(4, 16);
#undef LPD_CD_LAUNCH
    return hipGetLastError() == hipSuccess ? LPD_OK : LPD_ERR_HIP;
}

}  // extern "C"
