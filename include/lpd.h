/*
 * lpd.h -- C ABI of the MI355X (gfx950) low-rank stage of the LPD-SVM solver
 * (T. Glasmachers, "Recipe for Fast Large-scale SVM Training: Polishing,
 * Parallelism, and more RAM!").
 *
 * The library computes, on one GPU, the hot path of the method's two stages:
 *
 *   stage 1, Figure 1 step 1d:  G = Z W^T,  Z[i,b] = exp(-gamma ||x_i - l_b||^2)
 *   stage 2, Figure 1 step 2a:  m_i = G_i w
 *
 * plus the one-off host preparation of steps 1a-1c (landmark kernel matrix,
 * symmetric eigendecomposition, inverse-square-root factor with small
 * components dropped, Section 4).
 *
 * Symbols.  The paper calls the B x B factor of step 1c "L = U sqrt(D^-1)" and
 * sets G = Z L.  This interface stores its transpose W = sqrt(D^-1) U^T, one
 * whitened direction per ROW (r rows of length B, r <= B the number of kept
 * components), so that G = Z W^T and both products on the device contract
 * over the contiguous axis of two row-major operands.  "L" in this header is
 * the B x d matrix of landmark points (the random subset of step 1a).
 *
 * Conventions for every call.
 *   - All matrices are row-major fp32 with an explicit leading dimension
 *     (elements, >= number of columns).
 *   - "device" pointers are HIP device memory of the current device, owned by
 *     the caller (e.g. torch tensors); "host" pointers are ordinary memory.
 *     Device matrix pointers and leading dimensions need no alignment, but the
 *     fast path needs 16-byte aligned pointers and leading dimensions that are
 *     multiples of 4; anything else takes a slower element-wise loader.
 *   - Device calls only enqueue work on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return; results are ready once the
 *     stream has been synchronised.  The library allocates no device memory.
 *   - Sizes may be zero: the call then does nothing and returns LPD_OK.
 *   - Every function returns an lpd_status; nothing throws or exits.
 *     Execution faults of an enqueued kernel surface at the caller's next
 *     synchronisation, launch failures are returned as LPD_ERR_HIP.
 *   - Inputs and outputs must not overlap.
 *
 * Accuracy of the kernel block.  The device evaluates the squared distance of
 * the Gaussian kernel (Section 5) as ||x-c||^2 + ||l-c||^2 - 2 (x-c).(l-c) in
 * fp32, with the origin c at the mean of (a sample of) the landmarks, so that a
 * constant offset of the features costs no accuracy, and clamps it at 0.  Its
 * rounding error grows with the spread of the data around c, not with the
 * distance: |error of gamma * dist| <~ 2^-22 * gamma * (||x-c||^2 + ||l-c||^2),
 * and the same relative error appears in Z[i,b].  Measured against double
 * precision: 1e-7 relative Frobenius error of Z while gamma * ||x-c||^2 is of
 * order 1 (all of this project's workloads, also with features offset by 30 or
 * 1000 standard deviations, and 8-bit pixel values with gamma = 2^-22), 7e-6 for
 * two clusters 60 standard deviations apart (gamma * ||x-c||^2 about 30), where
 * the factor still meets its 1e-4.  Beyond gamma * ||x-c||^2 of about 1e2 for
 * the bulk of the points the 1e-4 of the factor is no longer assured; such data
 * has a kernel matrix close to the identity, and the fp32 factor degrades
 * gradually, it does not fail.  Kernel arguments gamma * dist beyond about 87
 * give exactly 0 in fp32 where double precision gives less than 1e-38.  The
 * gather route of the compressed-row entry points keeps the origin at 0 (sparse
 * rows stay sparse).
 */
#ifndef LPD_H
#define LPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LPD_OK = 0,
    LPD_ERR_NULL = -1,      /* a required pointer is NULL                       */
    LPD_ERR_SHAPE = -2,     /* negative size, r > B, or a size above the limits */
    LPD_ERR_LD = -3,        /* a leading dimension is smaller than the row      */
    LPD_ERR_WORKSPACE = -4, /* workspace missing, misaligned or too small       */
    LPD_ERR_HIP = -5,       /* a HIP runtime call or kernel launch failed       */
    LPD_ERR_NUMERIC = -6,   /* eigensolver did not converge / kernel matrix not
                               positive (largest eigenvalue <= 0)               */
    LPD_ERR_LIMIT = -7      /* lpd_predict_noalloc only: the shape needs more
                               than its fixed scratch                           */
} lpd_status;

/* Library version, major * 100 + minor. */
int lpd_version(void);

/* Static description of a status code (never NULL). */
const char *lpd_strerror(int status);

/*
 * Process-wide tuning knobs (not part of the method; defaults are chosen per
 * shape).  The only state the library keeps besides the scratch of
 * lpd_predict_noalloc.  Each is an atomic integer: it may be set at any time
 * from any thread; a call that is running reads it once per kernel launch, so a
 * change takes effect from the next launch on (results do not depend on them
 * beyond rounding, see the tile-independence tests).
 *   LPD_OPT_GEMM_TILE  workgroup tile of the two MFMA products:
 *                      0 = choose by shape, 1 = 128x128, 2 = 256x128, 3 = 256x256, 4 = 64x128
 *   LPD_OPT_GEMM_PIPELINE  main-loop schedule of the MFMA products: 0 = plain load/compute/store,
 *                      1 = software-pipelined across the barrier, 2 (default) = as 1, and the
 *                      whitening product keeps two k-tiles in flight from memory instead of one,
 *                      products with at most 64 columns four, requested two at a time
 *                      (all three visit k in the same order: identical results)
 *   LPD_OPT_CSR_ROUTE  route of the compressed-row entry points: 0 (default) = by density,
 *                      1 = dense panels, 2 = gather; set it before the workspace query
 *   LPD_OPT_SMALL_PATH the factor for B <= 256 landmarks (and d <= 1024): 1 (default) = one
 *                      launch per call, the kernel block stays in LDS; 0 = the panel schedule
 *   LPD_OPT_WHITEN_DC  lpd_whiten for B >= 512: 1 (default) = the tridiagonal problem is torn in two,
 *                      the halves solved concurrently and merged on the device; 0 = one QL
 *                      iteration over the whole matrix
 *   LPD_OPT_FUSED_SCORES prediction with up to 16 classifiers: 1 (default) = the kernel block is multiplied by
 *                      the folded weights in the write-out of its own launch and never stored; 0 = a panel of it
 *                      is stored and swept
 *   LPD_OPT_SWEEP_GRID workgroups of a full margin sweep: 0 (default) = chosen by the row length,
 *                      1..65536 = that many (each takes rows in a grid-stride loop)
 *   LPD_OPT_WHITEN_UPPER  lpd_whiten's reduction to tridiagonal form: 1 (default) = reads and updates the
 *                      upper triangle of the trailing matrix only, 0 = the whole symmetric matrix
 * Errors: LPD_ERR_SHAPE for an unknown option or value.
 */
typedef enum { LPD_OPT_GEMM_TILE = 1, LPD_OPT_GEMM_PIPELINE = 2, LPD_OPT_CSR_ROUTE = 3,
               LPD_OPT_SMALL_PATH = 4, LPD_OPT_WHITEN_DC = 5, LPD_OPT_WHITEN_UPPER = 6,
               LPD_OPT_SWEEP_GRID = 7, LPD_OPT_FUSED_SCORES = 8 } lpd_option;
int lpd_set_option(int option, int64_t value);

/*
 * Host preparation, Figure 1 steps 1a-1c with the dropping rule of Section 4
 * (second bullet).  Runs on the calling host in double precision, blocking.
 *
 *   K_LL[a,b] = exp(-gamma ||l_a - l_b||^2)                        (1a, Section 5 kernel)
 *   K_LL = U D U^T, eigenvalues sorted descending                  (1b)
 *   r = #{ j : D_j >= clip_ratio * D_0 and D_j > 0 }
 *   W[j,:] = D_j^-1/2 u_j^T  for j < r, rows r..B-1 are zero       (1c)
 *
 * Each kept eigenvector's sign makes its largest-magnitude entry positive
 * (first such entry on ties).  Section 4 (second bullet) ties the threshold to
 * machine precision relative to the largest eigenvalue and names no constant;
 * callers pass it, 1e-10 in this project's workloads.
 *
 *   L_host   in   B x d landmarks, leading dimension ldl
 *   W_host   out  B x B, leading dimension ldw
 *   eig_host out  B eigenvalues, descending (may be NULL)
 *   rank     out  r
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE, LPD_ERR_LD, LPD_ERR_NUMERIC.
 */
int lpd_whiten_host(const float *L_host, int64_t B, int64_t d, int64_t ldl,
                    double gamma, double clip_ratio,
                    float *W_host, int64_t ldw, double *eig_host, int64_t *rank);

/*
 * Figure 1 steps 1a-1c with the O(B^3) work on the device: the same result as
 * lpd_whiten_host (same definition, same ordering, clipping and sign rule),
 * computed in double precision by HIP kernels: kernel matrix of the landmarks,
 * Householder reduction to tridiagonal form, accumulation of the reflectors,
 * eigendecomposition of the tridiagonal matrix, scaling to W.  From 512
 * landmarks on the tridiagonal matrix is torn into 2, 4 or 8 pieces (from 512 /
 * 2,048 / 8,192 landmarks); each piece is solved by a QL iteration whose scalar
 * recurrence runs on a host thread of its own while the device applies its
 * plane rotations, and the pieces are merged on the device (secular equation,
 * deflation, a double-precision matrix product).  Eigenvectors of a repeated
 * eigenvalue may differ from the host routine's by a rotation within their
 * eigenspace.  The result is deterministic (no atomics anywhere).
 *
 *   L          device in   B x d floats, ldl
 *   W          device out  B x B floats, ldw; rows >= *rank are zero
 *   eig_host   host out    B doubles, descending; may be NULL
 *   rank       host out
 *   workspace  device, 256-byte aligned, at least lpd_whiten_workspace(B) bytes
 *              (two B x B double matrices, a third from 512 landmarks on, and
 *              vectors: 6.6 GB at B = 16,384)
 *   phase_seconds  host out, may be NULL: 5 doubles, wall time of the kernel
 *              matrix, the tridiagonalisation, the reflector accumulation, the
 *              eigendecomposition of the tridiagonal matrix (QL iterations with
 *              their rotation passes, and the merges), and the final scaling.
 *              Asking for them drains the stream between phases.
 * The call BLOCKS until W is complete.  It allocates no device memory.  At its
 * first call in a process (and again only for a larger B) it allocates
 * page-locked host staging (64 bytes per landmark plus up to 16 rotation buffers
 * of 256 B bytes each) and 17 events, which it keeps until the process ends; calls
 * from several threads are serialised on that staging.  B <= 46340.
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE, LPD_ERR_LD, LPD_ERR_WORKSPACE,
 * LPD_ERR_HIP, LPD_ERR_NUMERIC (QL did not converge, or no positive eigenvalue).
 */
int lpd_whiten_workspace(int64_t B, size_t *bytes);
int lpd_whiten(const float *L, int64_t B, int64_t d, int64_t ldl,
               double gamma, double clip_ratio,
               float *W, int64_t ldw, double *eig_host, int64_t *rank,
               void *workspace, size_t workspace_bytes, void *hip_stream,
               double *phase_seconds);

/*
 * Device scratch for lpd_nystrom_factor / lpd_kernel_block: squared row norms
 * of X and L plus one row panel of the kernel block Z.  `*bytes` receives the
 * recommended size for this shape; any 256-byte aligned buffer of at least
 * `*min_bytes` (may be NULL) works, larger ones allow larger panels.
 */
int lpd_nystrom_factor_workspace(int64_t n, int64_t d, int64_t B,
                                 size_t *bytes, size_t *min_bytes);

/*
 * Figure 1 step 1d on the device:  G[i, j] = sum_b W[j,b] * Z[i,b]  for j < r,
 * G[i, j] = 0 for r <= j < B, with Z[i,b] = exp(-gamma ||x_i - l_b||^2)
 * (Gaussian kernel of Section 5).  The n x B block Z is produced panel by
 * panel into the workspace and consumed at once; it never exists as a whole.
 * With B <= 256 landmarks (and d <= 1024) the whole step is one kernel launch
 * that keeps its rows of Z in LDS; the workspace is checked but not used.
 *
 *   X  device in   n x d, ldx          L  device in   B x d, ldl
 *   W  device in   r x B, ldw          G  device out  n x B, ldg
 *   workspace      device, 256-byte aligned, see lpd_nystrom_factor_workspace
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE, LPD_ERR_LD, LPD_ERR_WORKSPACE, LPD_ERR_HIP.
 */
int lpd_nystrom_factor(const float *X, int64_t n, int64_t d, int64_t ldx,
                       const float *L, int64_t B, int64_t ldl,
                       float gamma,
                       const float *W, int64_t r, int64_t ldw,
                       float *G, int64_t ldg,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Per-call device timing filled by lpd_nystrom_factor_profiled (milliseconds
 * summed over the launches of each kernel, from HIP events on `hip_stream`).
 * "norms" are the origin and the two row-norm kernels (3 launches).  The
 * one-launch path for B <= 256 books its single launch under "whiten" and
 * reports panel_rows = n. */
typedef struct {
    int32_t launches_norms, launches_kernel_block, launches_whiten;
    int32_t panel_rows;
    float ms_norms, ms_kernel_block, ms_whiten;
} lpd_factor_profile;

/*
 * Same work as lpd_nystrom_factor, with a HIP event recorded on `hip_stream`
 * before and after every kernel launch.  Unlike the plain call it BLOCKS until
 * the stream has drained, then fills *profile (host).  Meant for benchmarks.
 */
int lpd_nystrom_factor_profiled(const float *X, int64_t n, int64_t d, int64_t ldx,
                                const float *L, int64_t B, int64_t ldl,
                                float gamma,
                                const float *W, int64_t r, int64_t ldw,
                                float *G, int64_t ldg,
                                void *workspace, size_t workspace_bytes, void *hip_stream,
                                lpd_factor_profile *profile);

/*
 * Streaming form of step 1d for a factor that fits host memory but not device
 * memory (Section 4, "Algorithm Overview": every stage must be able to work in
 * chunks).  X, L and W stay on the device; G is produced chunk_rows rows at a
 * time into one of two device chunk buffers and copied to G_host on a second
 * stream of default priority while the next chunk is computed, so the copy
 * over PCIe hides behind the MFMA work whenever it is the shorter of the two.
 * Rows of G_host equal what lpd_nystrom_factor writes for the same row of X.
 *
 *   X, L, W     device in, as for lpd_nystrom_factor
 *   G_host      HOST out, n x B, ldg.  Page-locked memory (hipHostMalloc, a
 *               pinned torch tensor) is needed for the copies to overlap;
 *               pageable memory still gives the right result, serially.
 *   chunk_rows  rows per chunk, > 0 (the workspace query suggests a value)
 *   workspace   device, 256-byte aligned, at least the size the query returns
 *               for this chunk_rows: two chunk buffers and the factor scratch.
 * The call BLOCKS until G_host is complete.  It creates and destroys one stream
 * and four events; it allocates no device memory.
 * The query takes *chunk_rows in and out: a value <= 0 is replaced by the
 * suggested one (one kernel-block panel, at most n: short chunks keep the last,
 * exposed copy short); *bytes is the workspace size for the value it returns.
 * Errors: as lpd_nystrom_factor.
 */
int lpd_nystrom_factor_to_host_workspace(int64_t n, int64_t d, int64_t B,
                                         int64_t *chunk_rows, size_t *bytes);
int lpd_nystrom_factor_to_host(const float *X, int64_t n, int64_t d, int64_t ldx,
                               const float *L, int64_t B, int64_t ldl,
                               float gamma,
                               const float *W, int64_t r, int64_t ldw,
                               float *G_host, int64_t ldg, int64_t chunk_rows,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Step 1d, the kernel block and prediction for SPARSE inputs (Section 4: the
 * paper runs its kernel operations on sparse matrix products, since SVM data is
 * often sparse).  X is given in compressed-row form; L, W and the output are
 * dense as above.  Two routes, chosen by the density nnz / (n d):
 *   dense panels (8 % and above, or nnz unknown): each chunk of rows is written
 *     out into a dense panel in the workspace and goes through the same MFMA
 *     kernels as the dense entry points; a row's result equals that of the dense
 *     call on the written-out row;
 *   gather (below 8 %): the kernel block is accumulated entry by entry from the
 *     transposed landmarks (vector FMA), then consumed as in the dense schedule.
 *
 *   row_ptr    device in  n+1 offsets (int64), row i owns entries
 *                         row_ptr[i] .. row_ptr[i+1]-1; row_ptr[0] = 0
 *   col_idx    device in  column of each entry (int32), distinct within a row,
 *                         any order; an index outside [0, d) is ignored
 *   values     device in  value of each entry (float)
 *              col_idx and values may be NULL when there are no entries.
 *   nnz        number of stored entries (row_ptr[n]) if the caller knows it, else
 *              a negative value; it only selects the route (and, in the query,
 *              the workspace that route needs): pass the same value to both
 *   chunk_rows rows per panel, > 0 (the query suggests one: the factor's own
 *              panel size); *chunk_rows <= 0 on input asks for it
 *   workspace  device, 256-byte aligned, at least the query's size for this
 *              chunk_rows and nnz
 * Stream-ordered like the dense calls.  Errors: as lpd_nystrom_factor.
 */
int lpd_nystrom_factor_csr_workspace(int64_t n, int64_t d, int64_t B, int64_t nnz,
                                     int64_t *chunk_rows, size_t *bytes);
int lpd_nystrom_factor_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values,
                           int64_t n, int64_t d, int64_t nnz,
                           const float *L, int64_t B, int64_t ldl,
                           float gamma,
                           const float *W, int64_t r, int64_t ldw,
                           float *G, int64_t ldg, int64_t chunk_rows,
                           void *workspace, size_t workspace_bytes, void *hip_stream);
int lpd_kernel_block_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values,
                         int64_t n, int64_t d, int64_t nnz,
                         const float *L, int64_t B, int64_t ldl,
                         float gamma, float *Z, int64_t ldz, int64_t chunk_rows,
                         void *workspace, size_t workspace_bytes, void *hip_stream);
/* Scores of sparse new points: F = K(X, L) V^T as lpd_predict computes it (V c x B folded
 * classifiers, F n x c), X in compressed-row form as above; same workspace query. */
int lpd_predict_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *values,
                    int64_t n, int64_t d, int64_t nnz,
                    const float *L, int64_t B, int64_t ldl,
                    float gamma,
                    const float *V, int64_t c, int64_t ldv,
                    float *F, int64_t ldf, int64_t chunk_rows,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The kernel block alone (Figure 1 steps 1a / 1d, Section 5 kernel):
 * Z[i,b] = exp(-gamma ||x_i - l_b||^2), written in full to device memory.
 * With X = L this is the landmark kernel matrix K_LL of step 1a.
 *
 *   X device in n x d, ldx;  L device in B x d, ldl;  Z device out n x B, ldz
 *   workspace: 256-byte aligned, at least 4 n + 4 B + 4 d bytes with each of the three
 *   terms rounded up to 256 (row norms and the origin, see "Accuracy" above); the
 *   minimum lpd_nystrom_factor_workspace reports is always enough.
 */
int lpd_kernel_block(const float *X, int64_t n, int64_t d, int64_t ldx,
                     const float *L, int64_t B, int64_t ldl,
                     float gamma, float *Z, int64_t ldz,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Figure 1 step 2a for every row at once:  m[i] = sum_{j<r} G[i,j] * w[j].
 * Raw margins: no label, no offset (the method has no bias term, Section 2).
 *
 *   G device in n x r (ldg >= r);  w device in r;  m device out n
 */
int lpd_margins(const float *G, int64_t n, int64_t r, int64_t ldg,
                const float *w, float *m, void *hip_stream);

/*
 * Step 2a over a subset of rows, as the solver's shrinking re-check and
 * cross-validation folds need it (Section 4, "Shrinking" and
 * "Cross Validation"):  m[t] = sum_{j<r} G[rows[t], j] * w[j],  t < n_rows.
 *
 *   rows device in  n_rows int64 indices, each in [0, n).  The device checks them: an
 *                   index outside [0, n) reads nothing out of bounds and gives m[t] = NaN.
 * Errors: LPD_ERR_SHAPE also for n_rows > 0 with n = 0.
 */
int lpd_margins_rows(const float *G, int64_t n, int64_t r, int64_t ldg,
                     const int64_t *rows, int64_t n_rows,
                     const float *w, float *m, void *hip_stream);

/*
 * Step 2a for several weight vectors that share G (the classifiers of a C grid, of the folds, of the
 * class pairs; Section 4):  M[i, q] = sum_{j<r} G[i,j] * Ws[q,j],  q < k.
 * Up to 4 vectors are served by one pass over G with vector FMAs, more by the MFMA product G Ws^T on a
 * narrow tile, which reads G once as well (5 to 8 vectors take it when G, Ws, ldg, ldws and r allow 16-byte
 * loads, else the FMA pass).
 *   G device in n x r (ldg);  Ws device in k x r (ldws), one vector per row;  M device out n x k (ldm)
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE, LPD_ERR_LD, LPD_ERR_HIP.
 */
int lpd_margins_multi(const float *G, int64_t n, int64_t r, int64_t ldg,
                      const float *Ws, int64_t k, int64_t ldws,
                      float *M, int64_t ldm, void *hip_stream);

/*
 * Prediction (Section 4, "Algorithm Overview": the prediction step; Section 2: f(x) = <w, phi(x)>,
 * no offset).  A classifier trained on the rows of G has weights ws (r values); a new point x has
 * features W z(x), z(x)_b = exp(-gamma ||x - l_b||^2), so its score is ws . (W z(x)) = v . z(x) with
 * v = W^T ws folded once per classifier.
 *
 * lpd_fold_weights:  V[j, b] = sum_{k<r} Ws[j, k] * W[k, b]     (c x B)
 *   W device in r x B (ldw);  Ws device in c x r (ldws), one classifier per row;  V device out c x B (ldv)
 * lpd_predict:       F[i, j] = sum_b V[j, b] * exp(-gamma ||x_i - l_b||^2)     (n x c),  c <= B
 *   X device in n x d (ldx);  L device in B x d (ldl);  V device in c x B (ldv);  F device out n x c (ldf)
 *   workspace: as for lpd_nystrom_factor (lpd_nystrom_factor_workspace(n, d, B)).  Up to 64 classifiers the
 *   kernel block is contracted with V in the write-out of its own launch and never stored (the workspace
 *   holds per-tile shares of the scores); with more it is produced panel by panel and consumed at once by
 *   the MFMA product with V.
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE (incl. c > B), LPD_ERR_LD, LPD_ERR_WORKSPACE, LPD_ERR_HIP.
 */
int lpd_fold_weights(const float *W, int64_t r, int64_t B, int64_t ldw,
                     const float *Ws, int64_t c, int64_t ldws,
                     float *V, int64_t ldv, void *hip_stream);
int lpd_predict(const float *X, int64_t n, int64_t d, int64_t ldx,
                const float *L, int64_t B, int64_t ldl, float gamma,
                const float *V, int64_t c, int64_t ldv,
                float *F, int64_t ldf,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * lpd_predict for callers that may not allocate and have no workspace to pass:
 * code that runs under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same result and same stream-ordered
 * behaviour as lpd_predict, without the workspace: the row norms, the origin and
 * the panel of the kernel block live in a fixed 32 MiB array in device memory
 * that belongs to the library (one per GPU, present from the library's first
 * use on that GPU until the process ends).  The call allocates nothing, on the
 * host or on the device, and calls no allocating routine.
 *
 * Limit: the minimum workspace lpd_nystrom_factor_workspace(n, d, B) reports
 * must not exceed 32 MiB = 33,554,432 bytes, i.e. roughly
 * 4 n + 4 B + 4 d + 4 min(n, 256) (B + 16) <= 2^25; e.g. B <= 16,384 with up to
 * 4 million points per call, B = 30,000 with up to 600,000.  Beyond it the call
 * does nothing and returns LPD_ERR_LIMIT.  Nothing in the array has to start at
 * zero; every call overwrites what it reads.
 * All calls on one GPU share the array: calls that may overlap on one GPU (two
 * streams, two host threads) race on it and give wrong scores; keep them on one
 * stream, or order them with events.
 * Errors: as lpd_predict (without LPD_ERR_WORKSPACE), and LPD_ERR_LIMIT.
 */
int lpd_predict_noalloc(const float *X, int64_t n, int64_t d, int64_t ldx,
                        const float *L, int64_t B, int64_t ldl, float gamma,
                        const float *V, int64_t c, int64_t ldv,
                        float *F, int64_t ldf, void *hip_stream);

/*
 * Squared norms of the rows of the factor, gsq[i] = sum_{j<r} G[i,j]^2: the
 * diagonal Q_ii of the dual problem (Section 2, equation (2)) that the
 * coordinate step divides by.  G device in n x r (ldg); gsq device out, n floats.
 */
int lpd_row_sqnorms(const float *G, int64_t n, int64_t r, int64_t ldg, float *gsq, void *hip_stream);

/* Result record of one binary problem of lpd_cd_solve. */
typedef struct {
    int64_t steps;        /* inner products spent: active steps, re-checks, final sweeps */
    int32_t epochs;       /* passes over the active list                               */
    int32_t converged;    /* 1: stopped by the rule below, 0: hit max_epochs            */
    int32_t active;       /* size of the active list at exit                            */
    float max_violation;  /* largest KKT violation seen in the last epoch               */
    float dual;           /* sum alpha - 1/2 ||w||^2                                    */
    int32_t reserved;
} lpd_cd_status;

/* Bytes of device scratch lpd_cd_solve needs (active / next / removed lists and counters). */
int lpd_cd_solve_workspace(int64_t n_problems, int64_t total_rows, size_t *bytes);

/*
 * Stage 2 of the method on the device: dual coordinate ascent with shrinking on
 * the rows of G, for a batch of independent binary problems that share G (grid
 * search over C, cross-validation folds, one-versus-one pairs; Section 4).
 * Per problem p (Section 2, equation (2); Figure 1 steps 2a-2b):
 *
 *   maximise sum_t alpha_t - 1/2 ||w||^2,  0 <= alpha_t <= C[p],
 *   w = sum_t alpha_t y_t g_{rows[t]},   t over the problem's listed rows;
 *   step on t: f = g.w;  alpha_t <- clip(alpha_t + (1 - y_t f)/||g||^2, 0, C);  w += d_alpha y_t g.
 *
 * Order, shrinking and stopping (Section 4, "Shrinking", fixes k = 5 and
 * eta = 5 %; the third bullet of the comparison with LLSVM in Section 4 names a
 * standard stopping criterion without spelling it out; the reading is this): round-robin over the active list, initially the listed order; a
 * variable whose step left alpha bit-for-bit unchanged shrink_k times in a row is
 * removed; after every round((1-eta)/eta) active steps one step is spent on the
 * oldest removed variable, which rejoins if the step changes it; when an epoch's
 * largest violation (max(grad,0) at 0, max(-grad,0) at C, |grad| inside, measured
 * before each step) is <= eps, w is recomputed from alpha (the incremental fp32
 * updates drift), all removed variables are swept with that w, violators
 * rejoin; the problem is done when there are none and the epoch itself had
 * started from a recomputed w.  shrink_k = 0
 * switches shrinking off, eta = 0 the interleaved re-checks.
 *
 *   G        device in   n x r (ldg), 1 <= r <= 16384.  With a 16-byte aligned G and ldg a
 *                        multiple of 4 rows are read 16 bytes at a time, also across column r
 *                        when r is not a multiple of 4: every row, the last included, must be
 *                        readable up to column 4 ceil(r / 4) (true for any matrix whose last
 *                        row is allocated to its full ldg, as lpd_nystrom_factor's output is)
 *   gsq      device in   n, from lpd_row_sqnorms
 *   prob_off device in   n_problems + 1 offsets into rows / y / alpha; prob_off[0] = 0,
 *                        non-decreasing, prob_off[n_problems] = total_rows
 *   rows     device in   total_rows indices into G, each in [0, n)
 *                        The host cannot see these two arrays; the device clamps offsets to
 *                        [0, total_rows] and indices to [0, n), so that wrong contents give
 *                        wrong solutions of the problems concerned, never an access outside
 *                        the arrays or G.
 *   y        device in   total_rows labels, +1 or -1
 *   C        device in   n_problems upper bounds
 *   alpha    device i/o  total_rows; start values (zeros, or a warm start) in, solution out
 *   w        device out  n_problems x r (ldw)
 *   status   device out  n_problems records
 * One workgroup per problem; problems run concurrently.  Calls with the same
 * alpha / workspace must not overlap.
 * Errors: LPD_ERR_NULL, LPD_ERR_SHAPE (incl. r > 16384, r = 0 or n = 0 with rows listed,
 * shrink_k > 255, eta outside [0,1)),
 * LPD_ERR_LD (ldg < r, ldw < r), LPD_ERR_WORKSPACE, LPD_ERR_HIP.
 */
int lpd_cd_solve(const float *G, int64_t n, int64_t r, int64_t ldg, const float *gsq,
                 int64_t n_problems, const int64_t *prob_off, int64_t total_rows,
                 const int64_t *rows, const float *y, const float *C,
                 float *alpha, float *w, int64_t ldw, lpd_cd_status *status,
                 float eps, int32_t max_epochs, int32_t shrink_k, float eta,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LPD_H */
