// Robust PCA by the inexact augmented Lagrange multiplier method (Alg. 3 and the
// low-rank + sparse decomposition problem of Sec. 5):
// the elementwise kernels around the randomized SVD.  All of them are single sweeps over
// m x n fp32 arrays (HBM-bound); the rank-l product L = U diag(shrunk sigma) V^T is
// recomputed inside the fused update instead of being stored and re-read.
#include <algorithm>

#include "common.h"

namespace brsvd {

constexpr int kRpcaBlocks = 1024;     // fixed grid of the reductions (deterministic partial sums)

__device__ __forceinline__ double block_sum(double v, double* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double s = 0.0;
  if (threadIdx.x == 0)
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += sh[w];
  return s;   // valid in thread 0
}

// part[2*b] = max |M| over the block's slice, part[2*b+1] = sum M^2.
template <typename T>
__global__ void __launch_bounds__(256)
k_rpca_norms(const T* __restrict__ M, int64_t count, double* __restrict__ part) {
  __shared__ double sh[4];
  __shared__ double shm[4];
  double mx = 0.0, ss = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
    const double v = (double)M[i];
    mx = fmax(mx, fabs(v));
    ss = fma(v, v, ss);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off, 64));
  if (lane == 0) shm[wave] = mx;
  const double s = block_sum(ss, sh);
  if (threadIdx.x == 0) {
    part[2 * blockIdx.x] = fmax(fmax(shm[0], shm[1]), fmax(shm[2], shm[3]));
    part[2 * blockIdx.x + 1] = s;
  }
}

// scal[0] = max over blocks of part[2b], scal[1] = sum of part[2b+1]: each of the 256 threads adds its
// blocks b = tid, tid + 256, ... in order, then the threads' sums are added in lane and wave order.
__global__ void __launch_bounds__(256)
k_rpca_norms_final(const double* __restrict__ part, int nblocks, double* __restrict__ scal) {
  __shared__ double sh[4];
  __shared__ double shm[4];
  double mx = 0.0, ss = 0.0;
  for (int b = threadIdx.x; b < nblocks; b += 256) { mx = fmax(mx, part[2 * b]); ss += part[2 * b + 1]; }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off, 64));
  if (lane == 0) shm[wave] = mx;
  const double s = block_sum(ss, sh);
  if (threadIdx.x == 0) {
    scal[0] = fmax(fmax(shm[0], shm[1]), fmax(shm[2], shm[3]));
    scal[1] = s;
  }
}

// out[blockIdx.x] = sum of part[blockIdx.x * per .. min(nblocks, (blockIdx.x + 1) * per)): thread t adds its
// entries t, t + 256, ... of the slice in order, then the threads' sums are added in lane and wave
// order.  One launch with per >= nblocks gives the whole sum; long lists take two launches.
__global__ void __launch_bounds__(256)
k_sum_partials(const double* __restrict__ part, int nblocks, int per, double* __restrict__ out) {
  __shared__ double sh[4];
  const int b0 = blockIdx.x * per, b1 = min(nblocks, b0 + per);
  double s = 0.0;
  for (int b = b0 + threadIdx.x; b < b1; b += 256) s += part[b];
  s = block_sum(s, sh);
  if (threadIdx.x == 0) out[blockIdx.x] = s;
}

// Multiplier initialisation of Alg. 3: Y0 = M / J, S0 = 0, and the first SVD input
// X0 = M - S0 + Y0 / mu0.
template <typename T>
__global__ void k_rpca_init(const T* __restrict__ M, int64_t count, T inv_J, T inv_mu,
                            T* __restrict__ Y, T* __restrict__ S, T* __restrict__ X) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const T mv = M[i];
  const T y = mv * inv_J;
  Y[i] = y;
  S[i] = T(0);
  X[i] = fma(y, inv_mu, mv);
}

template <typename T>
__device__ __forceinline__ T shrinkf(T x, T eps) {
  return x > eps ? x - eps : (x < -eps ? x + eps : T(0));
}

constexpr int kRpcaTR = 32;

// One ALM iteration after the SVD of X_i (the low-rank, sparse, multiplier and residual updates of
// Alg. 3, and the matrix handed to the SVD of the next iteration):
//   L = U diag(shrink(sigma, 1/mu)) V^T        (rank-l product, recomputed here, terms added in index order)
//   S = shrink(M - L + Y/mu, lambda/mu)
//   Z = M - L - S;  Y_out = Y_in + mu Z;  partial ||Z||_F^2
//   X_next = M - S + Y_out / mu_next
// Neither L nor S is stored by an iteration: nothing reads them before the loop ends, and leaving them out makes
// an iteration two reads (M, Y_in) and two writes (Y_out, X_next) per element.  The multiplier goes from one
// buffer to another, so that when the loop has ended the FINAL instance can repeat the last iteration's
// arithmetic on the multiplier that iteration read and store its L and S (and nothing else); Y_in may be the
// buffer L goes to (every thread reads its elements before it writes them).
//
// A lane moves 16 bytes (VW elements) of one row per access, at any element alignment (rows of odd length do
// not start on 16-byte boundaries); the lane that straddles the end of a row moves its elements one by one.  M
// and the multiplier are read and S, Y, X written with nontemporal accesses (each is touched once per
// iteration), and all loads of a lane are issued before the first value is used.  The threads of a workgroup
// form TR = threads / cvt row lanes of cvt vector columns each (cvt = 64, or the whole row when it has fewer
// than 64 vectors); a thread owns one vector column in the RPT rows tr, tr + TR, tr + 2 TR, ... of the tile,
// so the rows of V^T it multiplies are loaded once for all of them, and consecutive threads touch consecutive
// addresses: with 64 vector columns every memory instruction of a wave moves 1 KiB of one row, and a matrix of
// short rows (100 columns: 25 vectors, 20 row lanes) is walked as one contiguous stream instead of leaving
// most lanes of a 64-lane column tile idle.  The loads of M and of the multiplier are issued before the rows of U are
// staged, and the rows of V^T are fetched four at a time.  Eight waves of four rows each measured best on 76800 x 2000
// (with S still stored by every iteration, i.e. three writes: 581 us; four waves of eight rows 606 us, sixteen of
// two 619 us; one element per lane 664 us; a plain kernel with the same two reads and three writes per element
// reaches 5.4 TB/s = 570 us; without the store of S the kernel takes 476 us, with the loads hoisted 458 us, with
// line-aligned accesses 443 us; plain kernels with two reads and two writes per element: 401 us as one flat array,
// 456 us in this kernel's tiles, 434 us in the tiles with line-aligned accesses).
template <typename T, int WAVES, int RPT, bool STREAM, bool FINAL>
__global__ void __launch_bounds__(WAVES * 64)
k_rpca_update_vec(const T* __restrict__ M, const T* __restrict__ U, const T* __restrict__ sig,
                  const T* __restrict__ Vt, int64_t m, int64_t n, int l, T inv_mu, T mu,
                  T thr_s, T inv_mu_next, const T* Yin, T* Yout, T* __restrict__ X, T* Lout, T* __restrict__ S,
                  double* __restrict__ part, int cvt, int col_tiles, int line_shift) {
  extern __shared__ __align__(16) unsigned char us_raw[];
  T* us = reinterpret_cast<T*>(us_raw);
  __shared__ double sh[WAVES];
  constexpr int VW = 16 / (int)sizeof(T);
  constexpr int NTHREADS = WAVES * 64;
  typedef T vecT __attribute__((ext_vector_type(VW)));
  typedef vecT vecTu __attribute__((aligned(sizeof(T))));
  const int tid = threadIdx.x;
  const int TR = NTHREADS / cvt, tile_rows = TR * RPT;
  const int ct = blockIdx.x % col_tiles, rt = blockIdx.x / col_tiles;
  const int64_t row0 = (int64_t)rt * tile_rows;
  const int tr = tid / cvt, cv = tid - tr * cvt;
  // With 64 vector columns a wave moves 1 KiB of one row per access.  Rows whose pitch is not a whole number of
  // 128-byte lines start inside a line, and an access that starts inside a line shares its first and last line
  // with the neighbouring tiles' accesses (fetched and written twice by streaming accesses).  The rows of one
  // thread are TR = 8 apart, i.e. a whole number of lines when a row is a whole number of 16-byte vectors, so they
  // all start at the same offset within a line, and the wave shifts its columns left by that offset: every access
  // then starts on a line (76800 x 2000: 458 -> 436 us).  The host enables this when all four arrays sit at the
  // same offset within a line and has added the column tile the shift may need at the end of a row.
  const int delta = line_shift ? (int)(((uintptr_t)(M + (row0 + tr) * n) % 128) / sizeof(T)) : 0;
  const int64_t col = ((int64_t)ct * cvt + cv) * VW - delta;
  const int cnt = col < 0 ? 0 : (int)min((int64_t)VW, n - col);   // elements of this lane's vector inside the row
  const bool active = tr < TR && cnt > 0;
  // the lane's elements of M and of the multiplier are requested first: they are on their way while the tile's
  // rows of U are staged and while the rows of V^T are fetched
  vecT mv[RPT], yv[RPT], acc[RPT];
#pragma unroll
  for (int i = 0; i < RPT; ++i) { mv[i] = vecT{}; yv[i] = vecT{}; acc[i] = vecT{}; }
  if (active) {
    if (cnt == VW) {
#pragma unroll
      for (int i = 0; i < RPT; ++i) {
        const int64_t row = min(row0 + tr + (int64_t)TR * i, m - 1);
        if constexpr (STREAM) {
          mv[i] = __builtin_nontemporal_load((const vecTu*)(M + row * n + col));
          yv[i] = __builtin_nontemporal_load((const vecTu*)(Yin + row * n + col));
        } else {
          mv[i] = *(const vecTu*)(M + row * n + col);
          yv[i] = *(const vecTu*)(Yin + row * n + col);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < RPT; ++i) {
        const int64_t row = min(row0 + tr + (int64_t)TR * i, m - 1);
#pragma unroll
        for (int c = 0; c < VW; ++c)
          if (c < cnt) { mv[i][c] = M[row * n + col + c]; yv[i][c] = Yin[row * n + col + c]; }
      }
    }
  }
  for (int idx = tid; idx < tile_rows * l; idx += NTHREADS) {
    const int i = idx / l, t = idx - i * l;
    const int64_t row = row0 + i;
    const T sv = fmax(sig[t] - inv_mu, T(0));      // shrinkage of a non-negative singular value
    us[idx] = row < m ? U[row * l + t] * sv : T(0);
  }
  __syncthreads();
  double z2 = 0.0;
  if (active) {
    // rank-l product, terms added in index order; the rows of V^T are fetched four at a time so that their
    // latencies overlap
    const T* vp = Vt + col;
    auto load_v = [&](int t) -> vecT {
      if (cnt == VW) return *(const vecTu*)(vp + (int64_t)t * n);
      vecT v = vecT{};
#pragma unroll
      for (int c = 0; c < VW; ++c)
        if (c < cnt) v[c] = vp[(int64_t)t * n + c];
      return v;
    };
    auto add_term = [&](int t, const vecT& v) {
#pragma unroll
      for (int i = 0; i < RPT; ++i) {
        const T u = us[(tr + TR * i) * l + t];
#pragma unroll
        for (int c = 0; c < VW; ++c) acc[i][c] = fma(u, v[c], acc[i][c]);
      }
    };
    int t = 0;
    for (; t + 4 <= l; t += 4) {
      const vecT v0 = load_v(t), v1 = load_v(t + 1), v2 = load_v(t + 2), v3 = load_v(t + 3);
      add_term(t, v0); add_term(t + 1, v1); add_term(t + 2, v2); add_term(t + 3, v3);
    }
    for (; t < l; ++t) add_term(t, load_v(t));
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int64_t row = row0 + tr + (int64_t)TR * i;
      if (row < m) {
        vecT sv, yn, xn;
#pragma unroll
        for (int c = 0; c < VW; ++c) {
          const T lv = acc[i][c];
          sv[c] = shrinkf(fma(yv[i][c], inv_mu, mv[i][c] - lv), thr_s);
          const T z = mv[i][c] - lv - sv[c];            // zero in the components beyond the row's end
          yn[c] = fma(mu, z, yv[i][c]);
          xn[c] = fma(yn[c], inv_mu_next, mv[i][c] - sv[c]);
          z2 = fma((double)z, (double)z, z2);
        }
        const int64_t e = row * n + col;
        if (cnt == VW) {
          if constexpr (FINAL) {
            if constexpr (STREAM) __builtin_nontemporal_store(sv, (vecTu*)(S + e));
            else *(vecTu*)(S + e) = sv;
            *(vecTu*)(Lout + e) = acc[i];
          } else if constexpr (STREAM) {
            __builtin_nontemporal_store(yn, (vecTu*)(Yout + e));
            __builtin_nontemporal_store(xn, (vecTu*)(X + e));
          } else {
            *(vecTu*)(Yout + e) = yn;
            *(vecTu*)(X + e) = xn;
          }
        } else {
#pragma unroll
          for (int c = 0; c < VW; ++c)
            if (c < cnt) {
              if constexpr (FINAL) { S[e + c] = sv[c]; Lout[e + c] = acc[i][c]; }
              else { Yout[e + c] = yn[c]; X[e + c] = xn[c]; }
            }
        }
      }
    }
  }
  if constexpr (!FINAL) {
    const double s = block_sum(z2, sh);
    if (tid == 0) part[blockIdx.x] = s;
  }
}

// P *= 1 / sqrt(*s2)  (normalisation of a power-method vector held in a padded panel)
template <typename T>
__global__ void k_scale_rsqrt(T* __restrict__ P, int64_t count, const double* __restrict__ s2) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const double v = *s2;
  P[i] = v > 0.0 ? (T)((double)P[i] / sqrt(v)) : T(0);
}

// Shape of the update kernel's workgroups for rows of n elements of esz bytes: vector columns per tile
// (64, or the whole row when it is shorter) and rows per tile.
constexpr int kRpcaUpdWaves = 8, kRpcaUpdRPT = 4;
struct RpcaUpdShape {
  int cvt, col_tiles, tile_rows;
};
static RpcaUpdShape rpca_update_shape(int64_t n, int esz) {
  const int vw = 16 / esz;
  const int64_t nvc = ceil_div(n, vw);
  RpcaUpdShape s;
  s.cvt = (int)std::min<int64_t>(64, nvc);
  s.col_tiles = (int)ceil_div(nvc, s.cvt);
  s.tile_rows = (kRpcaUpdWaves * 64 / s.cvt) * kRpcaUpdRPT;
  return s;
}

uint64_t rpca_part_doubles(int64_t m, int64_t n) {
  // the narrowest column tile any element type can take (64) bounds the number of partial sums
  const int64_t blocks = ceil_div(n, 64) * ceil_div(m, kRpcaTR);
  return (uint64_t)std::max<int64_t>(blocks + 64, 2 * kRpcaBlocks);   // + the first-level sums of the residual
}

template <typename T>
int rpca_norms(const T* M, int64_t count, double* part, double* scal, hipStream_t stream) {
  hipLaunchKernelGGL(k_rpca_norms<T>, dim3(kRpcaBlocks), dim3(256), 0, stream, M, count, part);
  hipLaunchKernelGGL(k_rpca_norms_final, dim3(1), dim3(256), 0, stream, part, kRpcaBlocks, scal);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T>
int rpca_init(const T* M, int64_t count, T inv_J, T inv_mu, T* Y, T* S, T* X, hipStream_t stream) {
  hipLaunchKernelGGL(k_rpca_init<T>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, stream, M, count, inv_J,
                     inv_mu, Y, S, X);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T, bool FINAL>
static int rpca_update_launch(const T* M, const T* U, const T* sig, const T* Vt, int64_t m, int64_t n, int l, T mu,
                              T lambda, T mu_next, const T* Yin, T* Yout, T* X, T* Lout, T* S, double* part,
                              int* nparts_out, hipStream_t stream) {
  if (m <= 0 || n <= 0 || l <= 0) return BRSVD_ERR_ARG;
  RpcaUpdShape sh = rpca_update_shape(n, (int)sizeof(T));
  constexpr int VW = 16 / (int)sizeof(T);
  // line-aligned accesses (see the kernel): whole vectors per row, 64 vector columns, all arrays at one offset
  // within a 128-byte line; the shift is at most 7 vectors, which may take one more column tile
  const uintptr_t a0 = (uintptr_t)M % 128;
  const bool same_line = FINAL ? ((uintptr_t)Yin % 128 == a0 && (uintptr_t)S % 128 == a0 && (uintptr_t)Lout % 128 == a0)
                               : ((uintptr_t)Yin % 128 == a0 && (uintptr_t)Yout % 128 == a0 && (uintptr_t)X % 128 == a0);
  const bool line_shift = sh.cvt == 64 && n % VW == 0 && a0 % 16 == 0 && same_line && (n * sizeof(T)) % 128 != 0;
  if (line_shift) sh.col_tiles = (int)ceil_div(ceil_div(n, VW) + 7, sh.cvt);
  const int64_t wgs = ceil_div(m, sh.tile_rows) * sh.col_tiles;
  if (wgs > INT32_MAX || (uint64_t)wgs + 64 > rpca_part_doubles(m, n)) return BRSVD_ERR_ARG;   // one partial sum per workgroup
  if (nparts_out) *nparts_out = (int)wgs;
  // the tile's rows of U: 32 x l elements with 64 vector columns; at most 32 KiB when rows are short (l <= n)
  const size_t lds = (size_t)sh.tile_rows * l * sizeof(T);
  constexpr int kMaxLds = 128 * 1024;
  if (lds > (size_t)kMaxLds) return BRSVD_ERR_ARG;
  // nontemporal accesses when every row starts on a 16-byte boundary; otherwise rows share their first and
  // last cache lines with their neighbours and plain accesses let the caches merge them
  const uintptr_t bits = FINAL ? ((uintptr_t)M | (uintptr_t)Yin | (uintptr_t)S | (uintptr_t)Lout)
                               : ((uintptr_t)M | (uintptr_t)Yin | (uintptr_t)Yout | (uintptr_t)X);
  const bool stream_ok = n % VW == 0 && bits % 16 == 0;
  auto kern = stream_ok ? k_rpca_update_vec<T, kRpcaUpdWaves, kRpcaUpdRPT, true, FINAL>
                        : k_rpca_update_vec<T, kRpcaUpdWaves, kRpcaUpdRPT, false, FINAL>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[stream_ok]) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds));
    attr_set[stream_ok] = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(kRpcaUpdWaves * 64), lds, stream, M, U, sig, Vt, m, n, l, T(1) / mu,
                     mu, lambda / mu, T(1) / mu_next, Yin, Yout, X, Lout, S, part, sh.cvt, sh.col_tiles, line_shift ? 1 : 0);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T>
int rpca_update(const T* M, const T* U, const T* sig, const T* Vt, int64_t m, int64_t n, int l, T mu, T lambda,
                T mu_next, const T* Yin, T* Yout, T* X, double* part, int* nparts_out, hipStream_t stream) {
  return rpca_update_launch<T, false>(M, U, sig, Vt, m, n, l, mu, lambda, mu_next, Yin, Yout, X, nullptr, nullptr, part,
                                      nparts_out, stream);
}

template <typename T>
int rpca_finalize(const T* M, const T* U, const T* sig, const T* Vt, int64_t m, int64_t n, int l, T mu, T lambda,
                  const T* Yin, T* Lout, T* S, hipStream_t stream) {
  return rpca_update_launch<T, true>(M, U, sig, Vt, m, n, l, mu, lambda, mu /* unused */, Yin, nullptr, nullptr, Lout, S,
                                     nullptr, nullptr, stream);
}

// *resid2_out = sum of the per-workgroup partial sums rpca_update left in `part`, in two levels when
// there are many (first-level sums go behind the partials); fixed order.
int rpca_residual_sum(double* part, int nparts, double* resid2_out, hipStream_t stream) {
  if (nparts > 8192) {
    const int groups = 64, per = (int)ceil_div(nparts, groups);
    hipLaunchKernelGGL(k_sum_partials, dim3(groups), dim3(256), 0, stream, part, nparts, per, part + nparts);
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(256), 0, stream, part + nparts, groups, groups, resid2_out);
  } else {
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(256), 0, stream, part, nparts, nparts, resid2_out);
  }
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T>
int scale_rsqrt(T* P, int64_t count, const double* s2, hipStream_t stream) {
  hipLaunchKernelGGL(k_scale_rsqrt<T>, dim3((unsigned)ceil_div(count, 256)), dim3(256), 0, stream, P, count, s2);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

#define BRSVD_RPCA_INSTANTIATE(T)                                                                                   \
  template int rpca_norms<T>(const T*, int64_t, double*, double*, hipStream_t);                                     \
  template int rpca_init<T>(const T*, int64_t, T, T, T*, T*, T*, hipStream_t);                                      \
  template int rpca_update<T>(const T*, const T*, const T*, const T*, int64_t, int64_t, int, T, T, T, const T*, T*, \
                              T*, double*, int*, hipStream_t);                                                      \
  template int rpca_finalize<T>(const T*, const T*, const T*, const T*, int64_t, int64_t, int, T, T, const T*, T*,  \
                                T*, hipStream_t);                                                                   \
  template int scale_rsqrt<T>(T*, int64_t, const double*, hipStream_t);
BRSVD_RPCA_INSTANTIATE(float)
BRSVD_RPCA_INSTANTIATE(double)
#undef BRSVD_RPCA_INSTANTIATE

}  // namespace brsvd
