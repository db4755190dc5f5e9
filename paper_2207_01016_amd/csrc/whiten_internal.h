// Pieces of the stage-1 preparation (Figure 1 steps 1b-1c) shared by the host routine and the device
// routine: the implicit-shift QL iteration on the tridiagonal matrix, which is serial scalar work and
// stays on the host in both, handing its plane rotations to the caller in batches of whole sweeps.
#pragma once
#include <cstddef>
#include <cstdint>
#include <functional>
#include <vector>

namespace lpd_host {

// One QL sweep: rotations with index i = hi down to lo (rotation i mixes eigenvector rows i and i+1);
// their (c, s) pairs sit at cs[off + 2*(hi - i)].
struct Sweep { int64_t lo, hi; size_t off; };

// The caller supplies the storage the (c, s) pairs of a batch are written to: `buffer` returns room for
// batch * 2 * n doubles (it may block until such a buffer is free again); `apply` then gets the sweeps of the
// batch, that same pointer and the number of doubles written.
using RotationBuffer = std::function<double *()>;
using ApplyRotations = std::function<void(const std::vector<Sweep> &, const double *, size_t)>;

// Eigenvalues of the symmetric tridiagonal matrix (dg, e; e[j] couples j and j+1) into dg.  Every
// `batch` sweeps the recorded rotations are passed to `apply`, in order, and forgotten.  `progress`
// (may be empty) is called with the number of eigenvalues found so far.  False if an eigenvalue
// needs more than 60 sweeps or `buffer` returns NULL.
bool tridiag_ql(double *dg, double *e, int64_t n, int batch, const RotationBuffer &buffer,
                const ApplyRotations &apply, const std::function<void(int64_t)> &progress);

// Descending order of the eigenvalues (stable) and the number r of leading ones that are positive and
// at least clip_ratio times the largest (step 1c).  eig_sorted may be NULL.
int64_t order_and_clip(const double *dg, int64_t n, double clip_ratio, std::vector<int64_t> &ord,
                       double *eig_sorted);

// Switch of the device routine: 1 (default) = matrices of 512 rows and more are torn in two, the halves solved
// by two concurrent QL iterations and merged on the device; 0 = one QL iteration over the whole matrix.
void set_divide_and_conquer(int on);
// 1 (default) = the Householder reduction reads and maintains the upper triangle of the trailing matrix only
// (half the bytes per column); 0 = the whole symmetric matrix.
void set_upper_triangle_pass(int on);

}  // namespace lpd_host
