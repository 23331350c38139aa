// SVD of the small l x l factor (Alg. 1 step 5 / Alg. 2 line 11) by one-sided (Hestenes) Jacobi.
//
// With B^T = W_B * R (thin QR of the n x l panel), R = Ur * diag(s) * Vr^T gives
// B = Vr * diag(s) * (W_B Ur)^T, i.e. the small left factor is Vr and V = W_B * Ur.
// The rows of a working copy of R are rotated in pairs until they are mutually orthogonal:
// J^T R = diag(s) Vr^T, so s_i is the norm of row i, Vr's column i the normalised row i, and
// Ur = J the accumulated rotations.  Everything is fp64; one workgroup of 1024 threads, each
// wave handling the row pairs of a round-robin step assigned to it.
#include "common.h"

namespace brsvd {

constexpr int kSvdThreads = 1024;
constexpr int kSvdWaves = kSvdThreads / 64;
constexpr int kMaxSweeps = 40;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// W: Lp x Lp working rows (stride Lp), JT: rows are the columns of J (stride Lp).
__global__ void __launch_bounds__(kSvdThreads)
k_jacobi(const double* __restrict__ R, int ldr, int l, int Lp, double* __restrict__ W,
         double* __restrict__ JT, double* __restrict__ sig, int* __restrict__ info,
         const int* __restrict__ breakdown_flag, double tol) {
  __shared__ int rotated;
  __shared__ int order[kMaxL];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (breakdown_flag && breakdown_flag[0] != 0) {
    if (tid == 0) { info[0] = 0; info[1] = 0; }
    return;
  }
  for (int idx = tid; idx < l * l; idx += kSvdThreads) {
    int i = idx / l, c = idx - i * l;
    W[(int64_t)i * Lp + c] = R[(int64_t)i * ldr + c];
    JT[(int64_t)i * Lp + c] = (i == c) ? 1.0 : 0.0;
  }
  const int L2 = (l + 1) & ~1;         // even number of players; index l is a phantom when l is odd
  const int npairs = L2 / 2;
  int sweeps = 0, converged = (l < 2);
  while (!converged && sweeps < kMaxSweeps) {
    if (tid == 0) rotated = 0;
    __syncthreads();
    for (int step = 0; step < L2 - 1; ++step) {
      for (int pi = wave; pi < npairs; pi += kSvdWaves) {
        int a, b;
        if (pi == 0) { a = L2 - 1; b = step; }
        else { a = (step + pi) % (L2 - 1); b = (step - pi + (L2 - 1)) % (L2 - 1); }
        if (a >= l || b >= l) continue;
        if (a > b) { int t = a; a = b; b = t; }
        double* wa = W + (int64_t)a * Lp;
        double* wb = W + (int64_t)b * Lp;
        double al = 0.0, be = 0.0, ga = 0.0;
        for (int e = lane; e < l; e += 64) {
          double x = wa[e], y = wb[e];
          al = fma(x, x, al); be = fma(y, y, be); ga = fma(x, y, ga);
        }
        al = wave_sum(al); be = wave_sum(be); ga = wave_sum(ga);
        if (fabs(ga) > tol * sqrt(al * be) && al > 0.0 && be > 0.0) {
          double zeta = (be - al) / (2.0 * ga);
          double t = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
          double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
          double* ja = JT + (int64_t)a * Lp;
          double* jb = JT + (int64_t)b * Lp;
          for (int e = lane; e < l; e += 64) {
            double x = wa[e], y = wb[e];
            wa[e] = c * x - s * y; wb[e] = s * x + c * y;
            double u = ja[e], v = jb[e];
            ja[e] = c * u - s * v; jb[e] = s * u + c * v;
          }
          if (lane == 0) rotated = 1;
        }
      }
      __syncthreads();
    }
    ++sweeps;
    converged = (rotated == 0);
    __syncthreads();
  }
  // singular values = row norms; rank them (descending, ties by index)
  for (int i = wave; i < l; i += kSvdWaves) {
    double s2 = 0.0;
    for (int e = lane; e < l; e += 64) { double x = W[(int64_t)i * Lp + e]; s2 = fma(x, x, s2); }
    s2 = wave_sum(s2);
    if (lane == 0) sig[Lp + i] = sqrt(s2);      // unsorted copy in the second half of sig
  }
  __syncthreads();
  for (int i = tid; i < l; i += kSvdThreads) {
    double si = sig[Lp + i];
    int rank = 0;
    for (int j = 0; j < l; ++j) {
      double sj = sig[Lp + j];
      rank += (sj > si) || (sj == si && j < i);
    }
    order[rank] = i;
  }
  __syncthreads();
  for (int i = tid; i < l; i += kSvdThreads) sig[i] = sig[Lp + order[i]];
  // reorder rows in place is awkward; publish the permutation instead (third part of sig, as doubles)
  for (int i = tid; i < l; i += kSvdThreads) sig[2 * Lp + i] = (double)order[i];
  if (tid == 0) { info[0] = sweeps; info[1] = converged; }
}

// Scatter the sorted factors: XV[kk][i] = W[o_i][kk] / s_i (Vr), XU[kk][i] = JT[o_i][kk] (Ur);
// fp32 zero-padded Lp x Lp operands for the lifts, and optional dense fp64 l x l copies.
__global__ void k_svd_outputs(const double* __restrict__ W, const double* __restrict__ JT,
                              const double* __restrict__ sig, int l, int Lp, double* __restrict__ S,
                              float* __restrict__ S32, float* __restrict__ XV, float* __restrict__ XU,
                              double* __restrict__ Ur, double* __restrict__ Vr) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= Lp * Lp) return;
  int kk = idx / Lp, i = idx - kk * Lp;
  float xv = 0.f, xu = 0.f;
  if (kk < l && i < l) {
    int o = (int)sig[2 * Lp + i];
    double s = sig[i];
    double v = s > 0.0 ? W[(int64_t)o * Lp + kk] / s : 0.0;
    double u = JT[(int64_t)o * Lp + kk];
    xv = (float)v; xu = (float)u;
    if (Vr) Vr[(int64_t)kk * l + i] = v;
    if (Ur) Ur[(int64_t)kk * l + i] = u;
    if (kk == 0) {
      if (S) S[i] = s;
      if (S32) S32[i] = (float)s;
    }
  }
  if (XV) XV[idx] = xv;
  if (XU) XU[idx] = xu;
}

int small_svd(const double* R, int ldr, int l, int Lp, SvdWork& w, const int* breakdown_flag, double* S,
              float* S32, float* XV, float* XU, double* Ur, double* Vr, hipStream_t stream) {
  if (l < 1 || l > kMaxL) return BRSVD_ERR_ARG;
  hipLaunchKernelGGL(k_jacobi, dim3(1), dim3(kSvdThreads), 0, stream, R, ldr, l, Lp, w.W, w.J, w.sig, w.info,
                     breakdown_flag, 1e-13);
  BRSVD_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_svd_outputs, dim3((unsigned)ceil_div((int64_t)Lp * Lp, 256)), dim3(256), 0, stream, w.W,
                     w.J, w.sig, l, Lp, S, S32, XV, XU, Ur, Vr);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

}  // namespace brsvd
