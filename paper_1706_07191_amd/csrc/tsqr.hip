// TSQR route of the panel orthonormaliser: the fallback taken when CholeskyQR breaks down
// (Gram matrix numerically singular), and selectable with BRSVD_ORTH_TSQR.
//
// The triangular factor R of the tall panel P is computed by a tree of Householder QR
// factorisations in fp64 (row chunks of 1024 rows are factored independently, their l x l
// factors are stacked and factored again until one remains) -- the reduction tree of the
// communication-avoiding QR the paper orthonormalises with (Sec. 3 "Orthonormalization").
// No Gram matrix is formed, so cond(P) is not squared.  The orthonormal factor is then
// obtained as Q = P R^-1 (one thin GEMM) followed by one CholeskyQR sweep that removes the
// eps32 * cond(P) loss of orthogonality of that product.  Diagonal entries of R below
// 1e-7 |R|_max (pure rounding noise of an fp32 panel) are clamped to that value so that
// R^-1 stays finite; the affected columns of Q are then arbitrary directions, which is all a
// numerically rank-deficient panel determines.
#include "common.h"

namespace brsvd {

constexpr int kTsqrC = 1024;   // rows per chunk (>= kMaxL so that every chunk yields a full l x l factor)

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Householder QR of one chunk of rows of src (row-major, leading dimension lds_, l columns,
// element type T).  work: per-chunk column-major fp64 scratch (Lp columns of kTsqrC rows).
// The chunk's l x l upper-triangular factor goes to rows [chunk*l, chunk*l + l) of dst
// (row-major fp64, leading dimension Lp).
template <typename T>
__global__ void __launch_bounds__(1024)
k_tsqr_chunk(const T* __restrict__ src, int64_t rows, int64_t lds_, int l, int Lp,
             double* __restrict__ work, double* __restrict__ dst) {
  __shared__ double red[16];
  __shared__ double hv[2];          // [0] = beta, [1] = alpha (the new diagonal entry)
  __shared__ double diag[kMaxL];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t r0 = (int64_t)blockIdx.x * kTsqrC;
  const int rc = (int)min((int64_t)kTsqrC, rows - r0);
  double* wk = work + (int64_t)blockIdx.x * kTsqrC * Lp;
  for (int idx = tid; idx < kTsqrC * l; idx += 1024) {
    const int row = idx / l, c = idx - row * l;
    wk[(int64_t)c * kTsqrC + row] = row < rc ? (double)src[(r0 + row) * lds_ + c] : 0.0;
  }
  __syncthreads();
  for (int j = 0; j < l; ++j) {
    double* vj = wk + (int64_t)j * kTsqrC;
    // norm of column j below (and including) the diagonal
    double p = 0.0;
    for (int r = j + tid; r < kTsqrC; r += 1024) p = fma(vj[r], vj[r], p);
    p = wave_sum_d(p);
    if (lane == 0) red[wave] = p;
    __syncthreads();
    if (tid == 0) {
      double nrm2 = 0.0;
      for (int w = 0; w < 16; ++w) nrm2 += red[w];
      const double x0 = vj[j];
      const double nrm = sqrt(nrm2);
      const double alpha = x0 > 0.0 ? -nrm : nrm;
      const double v0 = x0 - alpha;
      const double vnorm2 = nrm2 - x0 * x0 + v0 * v0;
      hv[0] = vnorm2 > 0.0 ? 2.0 / vnorm2 : 0.0;
      hv[1] = alpha;
      vj[j] = v0;
      diag[j] = alpha;
    }
    __syncthreads();
    const double beta = hv[0];
    // apply I - beta v v^T to the trailing columns, one column per wave at a time
    for (int c = j + 1 + wave; c < l; c += 16) {
      double* col = wk + (int64_t)c * kTsqrC;
      double w = 0.0;
      for (int r = j + lane; r < kTsqrC; r += 64) w = fma(vj[r], col[r], w);
      w = wave_sum_d(w) * beta;
      for (int r = j + lane; r < kTsqrC; r += 64) col[r] = fma(-w, vj[r], col[r]);
    }
    __syncthreads();
  }
  double* out = dst + (int64_t)blockIdx.x * l * Lp;
  for (int idx = tid; idx < l * l; idx += 1024) {
    const int i = idx / l, c = idx - i * l;
    out[(int64_t)i * Lp + c] = c > i ? wk[(int64_t)c * kTsqrC + i] : (c == i ? diag[i] : 0.0);
  }
}

// G <- R with the diagonal clamped away from zero (see the header comment).
__global__ void __launch_bounds__(1024)
k_tsqr_finish(const double* __restrict__ R, int l, int Lp, double* __restrict__ G) {
  __shared__ double dmax_sh;
  const int tid = threadIdx.x;
  if (tid == 0) {
    double d = 0.0;
    for (int i = 0; i < l; ++i) d = fmax(d, fabs(R[(int64_t)i * Lp + i]));
    dmax_sh = d;
  }
  __syncthreads();
  const double floor_ = 1e-7 * dmax_sh;
  for (int idx = tid; idx < l * l; idx += 1024) {
    const int i = idx / l, c = idx - i * l;
    double v = c >= i ? R[(int64_t)i * Lp + c] : 0.0;
    if (c == i && fabs(v) < floor_) v = v < 0.0 ? -floor_ : floor_;
    G[(int64_t)i * Lp + c] = v;
  }
}

static int64_t chunks_of(int64_t rows) { return ceil_div(rows, kTsqrC); }

uint64_t tsqr_work_bytes(int64_t rows, int Lp) {
  // chunk scratch of the largest level + two stacks of factors (ping-pong between levels)
  const int64_t c0 = chunks_of(rows);
  const uint64_t scratch = (uint64_t)c0 * kTsqrC * Lp * 8;
  const uint64_t stack = (uint64_t)c0 * Lp * Lp * 8;
  return scratch + 2 * stack + 1024;
}

template <typename T>
int tsqr_panel(T* P, T* tmp, int64_t rows, int l, int Lp, OrthWorkT<T>& w, double* Rtot, T** result,
               hipStream_t stream) {
  if (w.tsqr_bytes < tsqr_work_bytes(rows, Lp)) return BRSVD_ERR_BUDGET;
  const int64_t c0 = chunks_of(rows);
  double* scratch = (double*)w.tsqr_work;
  double* stack[2];
  stack[0] = scratch + (uint64_t)c0 * kTsqrC * Lp;
  stack[1] = stack[0] + (uint64_t)c0 * Lp * Lp;
  // level 0: the panel itself
  hipLaunchKernelGGL(k_tsqr_chunk<T>, dim3((unsigned)c0), dim3(1024), 0, stream, P, rows, (int64_t)Lp, l, Lp,
                     scratch, stack[0]);
  BRSVD_HIP_TRY(hipGetLastError());
  int cur = 0;
  int64_t nrows = c0 * l;         // stacked factor rows
  while (nrows > l) {
    const int64_t c = chunks_of(nrows);
    hipLaunchKernelGGL(k_tsqr_chunk<double>, dim3((unsigned)c), dim3(1024), 0, stream, stack[cur], nrows,
                       (int64_t)Lp, l, Lp, scratch, stack[cur ^ 1]);
    BRSVD_HIP_TRY(hipGetLastError());
    cur ^= 1;
    nrows = c * l;
  }
  // R (clamped) -> R^-1 -> Q1 = P R^-1 -> one CholeskyQR sweep
  hipLaunchKernelGGL(k_tsqr_finish, dim3(1), dim3(1024), 0, stream, stack[cur], l, Lp, w.G);
  BRSVD_HIP_TRY(hipGetLastError());
  double* Rt = stack[cur ^ 1];    // free now: keeps the TSQR factor for the product R2 * R
  BRSVD_TRY(chol_inv_factored<T>(w.G, l, Lp, Rt, w.Xinv, w.Rinv, w.flags, stream));
  BRSVD_TRY(gemm_an(P, Lp, rows, Lp, w.Rinv, Lp, tmp, Lp, Lp, w.gemm_scratch, w.gemm_scratch_bytes, stream));
  BRSVD_TRY(apply_to_companion<T>(w, Lp, stream));
  T* res = nullptr;
  BRSVD_TRY(cholqr_sweeps<T>(tmp, P, rows, l, Lp, 1, w, nullptr, &res, stream, true, Rtot != nullptr));
  *result = res;
  if (Rtot) BRSVD_TRY(triu_mul(w.R[0], Rt, l, Lp, Rtot, stream));
  return BRSVD_OK;
}

template int tsqr_panel<float>(float*, float*, int64_t, int, int, OrthWorkT<float>&, double*, float**, hipStream_t);
template int tsqr_panel<double>(double*, double*, int64_t, int, int, OrthWorkT<double>&, double*, double**,
                                hipStream_t);

}  // namespace brsvd
