// Internal declarations shared by the HIP translation units of libbrsvd (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "brsvd.h"

namespace brsvd {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int kMaxL = 512;       // largest sketch width l = k + p
constexpr int kTile = 16;        // MFMA tile edge (v_mfma_f32_16x16x4_f32)

// Padded panel width: every internal thin panel is rows x Lp, row-major, Lp a multiple of 16,
// columns l..Lp-1 kept at zero, so the GEMM kernels need no column masking on their inputs.
inline int padded_l(int l) { return (l + kTile - 1) / kTile * kTile; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

#define BRSVD_HIP_TRY(expr)                         \
  do {                                              \
    hipError_t e__ = (expr);                        \
    if (e__ != hipSuccess) return BRSVD_ERR_HIP;    \
  } while (0)

#define BRSVD_TRY(expr)                 \
  do {                                  \
    int s__ = (expr);                   \
    if (s__ != BRSVD_OK) return s__;    \
  } while (0)

// ---- thin-panel GEMMs (gemm_thin.hip) ------------------------------------------------------
// Optional events for per-kernel timing of one call: start/stop immediately around the MFMA kernel
// launch(es), sum_start/sum_stop around the split-sum kernels that follow (recorded even when there is
// nothing to sum).
struct KernelEvents {
  hipEvent_t start, stop, sum_start, sum_stop;
};

// Y (rows x ncols, ldy) = A (rows x K, lda) * X (K x Lp padded panel, ldx = Lp).
// scratch holds partial sums when the launch is split along K.  fp32 and fp64 (esz = element size).
uint64_t gemm_an_scratch_bytes(int64_t rows, int64_t K, int Lp, int esz = 4);
int gemm_an(const float* A, int64_t lda, int64_t rows, int64_t K, const float* X, int Lp,
            float* Y, int64_t ldy, int ncols, void* scratch, uint64_t scratch_bytes,
            hipStream_t stream, const KernelEvents* ev = nullptr);
int gemm_an(const double* A, int64_t lda, int64_t rows, int64_t K, const double* X, int Lp,
            double* Y, int64_t ldy, int ncols, void* scratch, uint64_t scratch_bytes,
            hipStream_t stream, const KernelEvents* ev = nullptr);

// Z (n x Lp padded panel) (+)= A^T * Q; A is rows x n (lda), Q is rows x Lp.  The row range is
// cut at multiples of block_rows (the row blocks of the method) and each block into equal
// sub-ranges; partial panels are summed in row order, so the result does not depend on timing.
uint64_t gemm_at_scratch_bytes(int64_t rows, int64_t n, int Lp, int64_t block_rows, int esz = 4);
int gemm_at(const float* A, int64_t lda, int64_t rows, int64_t n, const float* Q, int Lp,
            float* Z, bool accumulate, int64_t block_rows, void* scratch, uint64_t scratch_bytes,
            hipStream_t stream, const KernelEvents* ev = nullptr);
int gemm_at(const double* A, int64_t lda, int64_t rows, int64_t n, const double* Q, int Lp,
            double* Z, bool accumulate, int64_t block_rows, void* scratch, uint64_t scratch_bytes,
            hipStream_t stream, const KernelEvents* ev = nullptr);

// Launch plans as numbers (see brsvd_gemm_plan in the C ABI).
void gemm_an_plan_describe(int64_t rows, int64_t K, int Lp, int esz, int32_t out[12]);
void gemm_at_plan_describe(int64_t rows, int64_t n, int Lp, int64_t block_rows, int esz, int32_t out[12]);

// dst (rows x Lp, zero padded) <- src (rows x l dense)
int pad_panel(const float* src, int64_t rows, int l, float* dst, int Lp, hipStream_t stream);
int pad_panel(const double* src, int64_t rows, int l, double* dst, int Lp, hipStream_t stream);
// dst (rows x l dense) (+)= src (rows x Lp) restricted to the first l columns
int unpad_panel(const float* src, int64_t rows, int Lp, int l, float* dst, bool accumulate, hipStream_t stream);
int unpad_panel(const double* src, int64_t rows, int Lp, int l, double* dst, bool accumulate, hipStream_t stream);
// dst (l x rows, ld = rows) <- transpose of src (rows x Lp) restricted to the first l columns
int transpose_panel(const float* src, int64_t rows, int Lp, int l, float* dst, hipStream_t stream);
int transpose_panel(const double* src, int64_t rows, int Lp, int l, double* dst, hipStream_t stream);

// ---- orthonormalisation (orth.hip, tsqr.hip) -----------------------------------------------
// T = element type of the panels (float or double); the l x l factors are fp64 either way.
template <typename T>
struct OrthWorkT {
  double* gram_part;   // gram_chunks_max slots of Lp x Lp partial Gram sums (orth_gram_slots)
  int gram_chunks_max;
  double* G;           // Lp x Lp
  double* R[2];        // upper-triangular factors of the two CholeskyQR sweeps (stride Lp)
  double* Xinv;        // Lp x Lp fp64 scratch for R^-1
  T* Rinv;             // Lp x Lp zero-padded inverse factor in the panels' type (right operand of the apply GEMM)
  int* flags;          // device: [0] = breakdown flag (0 = none, else 1 + column)
  void* gemm_scratch;
  uint64_t gemm_scratch_bytes;
  void* tsqr_work;     // TSQR scratch
  uint64_t tsqr_bytes;
  // Optional companion panel (comp_rows x Lp): every R^-1 applied to the panel being orthonormalised
  // is applied to it as well (comp <- comp * R^-1, ping-ponging with comp_tmp; the result is in comp).
  T* comp = nullptr;
  T* comp_tmp = nullptr;
  int64_t comp_rows = 0;
};
typedef OrthWorkT<float> OrthWork;
// Applies the current w.Rinv to the companion panel, if any.
template <typename T> int apply_to_companion(OrthWorkT<T>& w, int Lp, hipStream_t stream);
uint64_t orth_gram_slots(int64_t rows, int Lp);   // Lp x Lp fp64 slots of partial Gram sums for such a panel
uint64_t tsqr_work_bytes(int64_t rows, int Lp);
// Orthonormalises the columns of P (rows x Lp padded panel, rows >= l).  tmp is a second
// rows x Lp buffer; *result is set to whichever of P / tmp holds the orthonormal panel.
// Rtot (stride Lp, fp64, may be null) receives the triangular factor with P_in = Q * Rtot.
// Asynchronous: a CholeskyQR breakdown is only reported through w.flags[0] on the device.
// final_basis = false: the panel only seeds the next power half step (one CholeskyQR sweep).
template <typename T>
int orth_panel(T* P, T* tmp, int64_t rows, int l, int Lp, int method, bool final_basis, OrthWorkT<T>& w,
               double* Rtot, T** result, hipStream_t stream);
// Pieces shared between the CholeskyQR and the Householder-tree routes (orth.hip, tsqr.hip).
template <typename T>
int cholqr_sweeps(T* P, T* tmp, int64_t rows, int l, int Lp, int nsweeps, OrthWorkT<T>& w, double* Rtot,
                  T** result, hipStream_t stream, bool strict_last, bool publish_R = false);
template <typename T>
int chol_inv_factored(double* G, int l, int Lp, double* Rout, double* Xtmp, T* Rinv, int* flags, hipStream_t stream);
template <typename T>
int tsqr_panel(T* P, T* tmp, int64_t rows, int l, int Lp, OrthWorkT<T>& w, double* Rtot, T** result,
               hipStream_t stream);
int triu_mul(const double* R2, const double* R1, int l, int Lp, double* Rtot, hipStream_t stream);
// *out (device) = min |R_ii| / max |R_ii| of the l x l triangular factor R (stride Lp)
int diag_ratio(const double* R, int l, int Lp, double* out, hipStream_t stream);

// ---- small SVD (small_svd.hip) -------------------------------------------------------------
struct SvdWork {
  double* W;     // Lp x Lp rows being orthogonalised
  double* J;     // Lp x Lp accumulated rotations (transposed)
  double* sig;   // 3 * Lp
  int* info;     // device: [0] sweeps, [1] converged
};
// R (l x l fp64, stride ldr): R = Ur diag(S) Vr^T.  Writes S (descending) as fp64 and/or in the
// panels' type TO, the zero-padded (Lp x Lp) operands XV = Vr and XU = Ur used by the lifts (type TO),
// and optional dense fp64 l x l Ur / Vr.  Skips the work when *breakdown_flag != 0.
template <typename TO>
int small_svd(const double* R, int ldr, int l, int Lp, SvdWork& w, const int* breakdown_flag,
              double* S, TO* S32, TO* XV, TO* XU, double* Ur, double* Vr, hipStream_t stream);

// ---- robust-PCA elementwise kernels (rpca.hip) ---------------------------------------------
// Number of doubles of partial-sum scratch the reductions below need.
uint64_t rpca_part_doubles(int64_t m, int64_t n);
// scal[0] = max |M_ij|, scal[1] = ||M||_F^2 (device doubles).  T = float or double throughout.
template <typename T> int rpca_norms(const T* M, int64_t count, double* part, double* scal, hipStream_t stream);
// Y0 = M * inv_J, S0 = 0, X0 = M - S0 + Y0 * inv_mu
template <typename T>
int rpca_init(const T* M, int64_t count, T inv_J, T inv_mu, T* Y, T* S, T* X, hipStream_t stream);
// Fused update after the SVD of X_i: with L = U diag(shrink(sig, 1/mu)) Vt (contraction over l) and
// S = shrink(M - L + Yin/mu, lambda/mu) formed in registers, writes Yout = Yin + mu (M - L - S), the next SVD input
// X = M - S + Yout/mu_next and per-workgroup partial sums of ||M-L-S||_F^2 into `part` (*nparts_out of them); L and
// S themselves are not stored.  U is m x l (ld l), Vt is l x n (ld n); Yout may be Yin.  rpca_residual_sum then adds
// the partial sums into *resid2_out in a fixed order.
template <typename T>
int rpca_update(const T* M, const T* U, const T* sig, const T* Vt, int64_t m, int64_t n, int l, T mu, T lambda,
                T mu_next, const T* Yin, T* Yout, T* X, double* part, int* nparts_out, hipStream_t stream);
int rpca_residual_sum(double* part, int nparts, double* resid2_out, hipStream_t stream);
// L and S of the iteration that used (U, sig, Vt, mu) and read the multiplier Yin, with the arithmetic of rpca_update.
// Lout may be Yin.
template <typename T>
int rpca_finalize(const T* M, const T* U, const T* sig, const T* Vt, int64_t m, int64_t n, int l, T mu, T lambda,
                  const T* Yin, T* Lout, T* S, hipStream_t stream);
// P[0..count) *= 1 / sqrt(*s2) (device scalar; a zero scalar zeroes P).
template <typename T> int scale_rsqrt(T* P, int64_t count, const double* s2, hipStream_t stream);

// ---- device-side Gaussian generator (philox.hip) -------------------------------------------
// Rows [row0, row0 + rows) of the m x l matrix Omega(seed) (Philox4x32-10 + Box-Muller, element
// e = row*l + col from output e&3 of counter e>>2) into out (rows x ld, columns l..ld-1 zeroed).
template <typename T>
int philox_normal(uint64_t seed, int64_t row0, int64_t rows, int l, T* out, int ld, hipStream_t stream);

// ---- machine probes (probe.hip) -------------------------------------------------------------
int probe(int kind, void* buf, uint64_t amount, double* seconds, double* work, hipStream_t stream);

}  // namespace brsvd
