// Orthonormalisation of tall thin panels (Alg. 1 step 3, Alg. 2 line 6) on gfx950.
//
// Main route: CholeskyQR applied twice.  G = P^T P is accumulated in fp64 (products of fp32
// values are exact in fp64), factored G = R^T R in fp64, and P <- P * R^-1 is one more thin
// GEMM on the MFMA path.  A pivot that falls below a relative threshold raises the breakdown
// flag; the caller then switches to the Householder-based TSQR route (tsqr.hip).
// The paper orthonormalises with a TSQR-based CAQR; range(P) -- all the method needs -- is the
// same for any orthonormalisation.
#include "common.h"

namespace brsvd {

template <typename T>
__global__ void k_reduce_splits_t(const T* __restrict__ part, int nsplit, int64_t split_stride,
                                  int64_t count, T* __restrict__ out) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= count) return;
  T s = T(0);
  for (int i = 0; i < nsplit; ++i) s += part[(int64_t)i * split_stride + idx];
  out[idx] = s;
}

// ---- Gram matrix -----------------------------------------------------------------------------
// grid = (row chunks, pairs (bi <= bj) of 64-column blocks); 256 threads, thread (ty, tx) owns
// the 4x4 entries G[64*bi + 4*ty + i][64*bj + 4*tx + j] of this chunk's partial sum.
constexpr int kGramRC = 32;

__global__ void __launch_bounds__(256)
k_gram(const float* __restrict__ P, int64_t rows, int Lp, int64_t rows_per_chunk,
       double* __restrict__ Gpart) {
  __shared__ float sI[kGramRC][64];
  __shared__ float sJ[kGramRC][64];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  // decode the block pair
  int nb = (Lp + 63) / 64;
  int bi = 0, rem = blockIdx.y;
  while (rem >= nb - bi) { rem -= nb - bi; ++bi; }
  const int bj = bi + rem;
  const int64_t rbeg = (int64_t)blockIdx.x * rows_per_chunk;
  const int64_t rend = min(rows, rbeg + rows_per_chunk);

  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

  for (int64_t r0 = rbeg; r0 < rend; r0 += kGramRC) {
    // kGramRC x 64 floats per operand = 512 float4, two per thread
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      int idx = tid + t * 256;
      int rr = idx >> 4, c4 = (idx & 15) * 4;
      int64_t row = r0 + rr;
      floatx4 vi = floatx4{0.f, 0.f, 0.f, 0.f}, vj = vi;
      if (row < rend) {
        if (bi * 64 + c4 < Lp) vi = *(const floatx4*)(P + row * Lp + bi * 64 + c4);
        if (bj * 64 + c4 < Lp) vj = *(const floatx4*)(P + row * Lp + bj * 64 + c4);
      }
      *(floatx4*)&sI[rr][c4] = vi;
      *(floatx4*)&sJ[rr][c4] = vj;
    }
    __syncthreads();
#pragma unroll 8
    for (int rr = 0; rr < kGramRC; ++rr) {
      floatx4 a = *(const floatx4*)&sI[rr][4 * ty];
      floatx4 b = *(const floatx4*)&sJ[rr][4 * tx];
      double bd[4] = {(double)b[0], (double)b[1], (double)b[2], (double)b[3]};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        double ad = (double)a[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(ad, bd[j], acc[i][j]);
      }
    }
    __syncthreads();
  }
  double* Go = Gpart + (int64_t)blockIdx.x * Lp * Lp;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int gi = bi * 64 + 4 * ty + i;
    if (gi < Lp) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int gj = bj * 64 + 4 * tx + j;
        if (gj < Lp) Go[(int64_t)gi * Lp + gj] = acc[i][j];
      }
    }
  }
}

// ---- Cholesky factor and its inverse ---------------------------------------------------------
// One workgroup of 1024 threads.  On entry the upper triangle of G (Lp x Lp, stride Lp) holds
// P^T P; on exit it holds R with G = R^T R.  X (Lp x Lp fp64 scratch) receives R^-1, which is
// also written as the zero-padded fp32 right operand of the apply GEMM.  A pivot <= tol * its
// original diagonal entry sets flag[0] = 1 + column index and ends the kernel.
__global__ void __launch_bounds__(1024)
k_chol_inv(double* __restrict__ G, int l, int Lp, double* __restrict__ Rout, double* __restrict__ X,
           float* __restrict__ Rinv32, int* __restrict__ flag, double tol) {
  __shared__ double d0[kMaxL];
  const int tid = threadIdx.x;
  const int ty = tid >> 5, tx = tid & 31;
  for (int i = tid; i < Lp * Lp; i += 1024) Rinv32[i] = 0.f;
  if (flag[0] != 0) return;   // an earlier panel already broke down: results are void anyway
  for (int i = tid; i < l; i += 1024) d0[i] = G[(int64_t)i * Lp + i];
  for (int j = 0; j < l; ++j) {
    __syncthreads();
    const double d = G[(int64_t)j * Lp + j];
    if (!(d > tol * d0[j])) {
      if (tid == 0) flag[0] = j + 1;
      return;
    }
    const double inv = 1.0 / sqrt(d);
    __syncthreads();
    for (int c = j + tid; c < l; c += 1024) G[(int64_t)j * Lp + c] *= inv;   // G[j][j] <- sqrt(d)
    __syncthreads();
    for (int rr = j + 1 + ty; rr < l; rr += 32) {
      const double f = G[(int64_t)j * Lp + rr];
      for (int c = rr + tx; c < l; c += 32) G[(int64_t)rr * Lp + c] -= f * G[(int64_t)j * Lp + c];
    }
  }
  __syncthreads();
  // R^-1 by back substitution, one column per thread: R X = I.
  for (int jj = tid; jj < l; jj += 1024) {
    X[(int64_t)jj * Lp + jj] = 1.0 / G[(int64_t)jj * Lp + jj];
    for (int i = jj - 1; i >= 0; --i) {
      double s = 0.0;
      for (int k = i + 1; k <= jj; ++k) s = fma(G[(int64_t)i * Lp + k], X[(int64_t)k * Lp + jj], s);
      X[(int64_t)i * Lp + jj] = -s / G[(int64_t)i * Lp + i];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < l * l; idx += 1024) {
    int i = idx / l, c = idx - i * l;
    double rv = c >= i ? G[(int64_t)i * Lp + c] : 0.0;
    Rout[(int64_t)i * Lp + c] = rv;
    if (c >= i) Rinv32[(int64_t)i * Lp + c] = (float)X[(int64_t)i * Lp + c];
  }
}

// Rtot = R2 * R1 (both upper triangular, l x l, stride Lp).
__global__ void k_triu_mul(const double* __restrict__ R2, const double* __restrict__ R1, int l, int Lp,
                           double* __restrict__ Rtot) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= l * l) return;
  int i = idx / l, c = idx - i * l;
  double s = 0.0;
  for (int k = i; k <= c; ++k) s = fma(R2[(int64_t)i * Lp + k], R1[(int64_t)k * Lp + c], s);
  Rtot[(int64_t)i * Lp + c] = s;
}

uint64_t orth_gram_chunks(int64_t rows) {
  int64_t c = ceil_div(rows, 1024);
  if (c > 64) c = 64;
  if (c < 1) c = 1;
  return (uint64_t)c;
}

static int gram(const float* P, int64_t rows, int Lp, OrthWork& w, hipStream_t stream) {
  int chunks = (int)orth_gram_chunks(rows);
  if (chunks > w.gram_chunks_max) return BRSVD_ERR_BUDGET;
  int64_t rpc = ceil_div(rows, chunks);
  rpc = ceil_div(rpc, kGramRC) * kGramRC;
  chunks = (int)ceil_div(rows, rpc);
  int nb = (Lp + 63) / 64;
  dim3 grid(chunks, nb * (nb + 1) / 2);
  hipLaunchKernelGGL(k_gram, grid, dim3(256), 0, stream, P, rows, Lp, rpc, w.gram_part);
  BRSVD_HIP_TRY(hipGetLastError());
  int64_t count = (int64_t)Lp * Lp;
  hipLaunchKernelGGL(k_reduce_splits_t<double>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, stream,
                     w.gram_part, chunks, count, count, w.G);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

int tsqr_panel(float* P, float* tmp, int64_t rows, int l, int Lp, OrthWork& w, double* Rtot,
               float** result, hipStream_t stream);

static int cholqr2(float* P, float* tmp, int64_t rows, int l, int Lp, OrthWork& w, double* Rtot,
                   float** result, hipStream_t stream) {
  const double tol = 1e-12;
  float* src = P;
  float* dst = tmp;
  for (int sweep = 0; sweep < 2; ++sweep) {
    BRSVD_TRY(gram(src, rows, Lp, w, stream));
    hipLaunchKernelGGL(k_chol_inv, dim3(1), dim3(1024), 0, stream, w.G, l, Lp, w.R[sweep], w.Xinv, w.Rinv,
                       w.flags, tol);
    BRSVD_HIP_TRY(hipGetLastError());
    BRSVD_TRY(gemm_an(src, Lp, rows, Lp, w.Rinv, Lp, dst, Lp, Lp, w.gemm_scratch, w.gemm_scratch_bytes, stream));
    float* t = src; src = dst; dst = t;
  }
  *result = src;   // after two swaps: the original P
  if (Rtot) {
    hipLaunchKernelGGL(k_triu_mul, dim3((unsigned)ceil_div((int64_t)l * l, 256)), dim3(256), 0, stream,
                       w.R[1], w.R[0], l, Lp, Rtot);
    BRSVD_HIP_TRY(hipGetLastError());
  }
  return BRSVD_OK;
}

int orth_panel(float* P, float* tmp, int64_t rows, int l, int Lp, int method, OrthWork& w, double* Rtot,
               float** result, hipStream_t stream) {
  if (rows < l) return BRSVD_ERR_ARG;
  if (method == BRSVD_ORTH_TSQR) return tsqr_panel(P, tmp, rows, l, Lp, w, Rtot, result, stream);
  return cholqr2(P, tmp, rows, l, Lp, w, Rtot, result, stream);
}

}  // namespace brsvd
