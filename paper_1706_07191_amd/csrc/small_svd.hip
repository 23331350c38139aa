// SVD of the small l x l factor (Alg. 1 step 5 / Alg. 2 line 11) by one-sided (Hestenes) Jacobi.
//
// With B^T = W_B * R (thin QR of the n x l panel), R = Ur * diag(s) * Vr^T gives
// B = Vr * diag(s) * (W_B Ur)^T, i.e. the small left factor is Vr and V = W_B * Ur.
// The rows of a working copy W of R are rotated in pairs (round-robin schedule) until they are
// mutually orthogonal: then W = diag(s) Vr^T, so s_i is the norm of row i and Vr's column i the
// normalised row i; Ur = R Vr diag(1/s) follows from one small product.  Everything is fp64.
//   l <= kJacobiLdsMaxL : one workgroup of 1024 threads, W resident in LDS for all sweeps.
//   larger l            : block Jacobi, one launch per round of block pairs, W in L2, block pairs in LDS.
#include <cstdlib>

#include "common.h"

namespace brsvd {

constexpr int kSvdThreads = 1024;
constexpr int kMaxSweeps = 40;
constexpr int kJacobiLdsMaxL = 128;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Pair pi of round-robin step `step` among L2 (even) players.
__device__ __forceinline__ void rr_pair(int pi, int step, int L2, int& a, int& b) {
  const int N = L2 - 1;
  if (pi == 0) { a = N; b = step; }
  else {
    a = step + pi; if (a >= N) a -= N;
    b = step - pi; if (b < 0) b += N;
  }
  if (a > b) { int t = a; a = b; b = t; }
}

// 1/sqrt(x) and 1/x for positive normal x: hardware seed plus two Newton steps (full fp64).
__device__ __forceinline__ double rsqrt_nr(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double h = 0.5 * x;
  y = fma(y, fma(-h * y, y, 0.5), y);
  y = fma(y, fma(-h * y, y, 0.5), y);
  return y;
}
__device__ __forceinline__ double rcp_nr(double x) {
  double y = __builtin_amdgcn_rcp(x);
  y = fma(y, fma(-x, y, 1.0), y);
  y = fma(y, fma(-x, y, 1.0), y);
  return y;
}

// Rotation (c, s) that makes two rows with squared norms al, be and inner product ga orthogonal:
// with zeta = (be - al) / (2 ga), t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)), c = 1/sqrt(1+t^2),
// s = c t, written so that it needs one reciprocal and two reciprocal square roots.
// Returns false (identity) when |ga| <= tol * sqrt(al * be).
// Sweeps end when a whole sweep met no pair with |cos| above kSettled: all cosines are then of the order
// l * kSettled^2 after that sweep's rotations (quadratic convergence), below the rotation threshold, so
// a further sweep that would only confirm it is not run.
// With results delivered in single precision the bar is lower: a last sweep whose largest cosine was below
// kSettledF32 leaves cosines of the order l * kSettledF32^2 = 1e-8, an order of magnitude below what the fp32
// lifts U = Q V_R and V = W_B U_R can show, and that saves one sweep of the seven to eight an l of 100 to 300 takes.
constexpr double kSettled = 1e-8;
constexpr double kSettledF32 = 1e-5;
__device__ __forceinline__ bool rotation(double al, double be, double ga, double tol2, double settled2, double& c,
                                         double& s, bool& big) {
  c = 1.0; s = 0.0;
  big = ga * ga > settled2 * al * be;
  if (!(ga * ga > tol2 * al * be)) return false;
  const double tau = be - al, g2 = 2.0 * ga;
  const double hh = fma(tau, tau, g2 * g2);
  const double h = hh * rsqrt_nr(hh);
  const double t = copysign(g2, g2 * tau >= 0.0 ? 1.0 : -1.0) * rcp_nr(fabs(tau) + h);
  c = rsqrt_nr(fma(t, t, 1.0));
  s = c * t;
  return true;
}

// Sum over the 16 lanes of a DPP row, result in every lane of the row.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, true);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_f64<0x128>(v);   // row_ror:8
  v += dpp_f64<0x124>(v);   // row_ror:4
  v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]
  return v;
}

// Singular values (row norms), their descending order, and the final rows, written to global.
template <int NTHREADS>
__device__ void publish(const double* W, int ld, int l, int Lp, double* Wg, double* sig, int* order_sh,
                        int tid, int lane, int wave) {
  for (int i = wave; i < l; i += NTHREADS / 64) {
    double s2 = 0.0;
    for (int e = lane; e < l; e += 64) { double x = W[(int64_t)i * ld + e]; s2 = fma(x, x, s2); }
    s2 = wave_sum(s2);
    if (lane == 0) sig[Lp + i] = sqrt(s2);
  }
  for (int i = tid; i < l; i += NTHREADS) order_sh[i] = 0;
  __syncthreads();
  for (int i = tid; i < l; i += NTHREADS) {
    const double si = sig[Lp + i];
    int rank = 0;
    for (int j = 0; j < l; ++j) {
      const double sj = sig[Lp + j];
      rank += (sj > si) || (sj == si && j < i);
    }
    order_sh[rank] = i;
  }
  __syncthreads();
  for (int i = tid; i < l; i += NTHREADS) {
    sig[i] = sig[Lp + order_sh[i]];
    sig[2 * Lp + i] = (double)order_sh[i];
  }
  if (Wg != W)
    for (int idx = tid; idx < l * l; idx += NTHREADS) {
      int i = idx / l, c = idx - i * l;
      Wg[(int64_t)i * Lp + c] = W[(int64_t)i * ld + c];
    }
}

// Sum over the 64 lanes of a wave, result in every lane: the four row sums are read as scalars and added.
__device__ __forceinline__ double lane_value(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave64_sum(double v) {
  v = row16_sum(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// Sum over groups of 8 lanes (half a DPP row), result in every lane of the group.
__device__ __forceinline__ double row8_sum(double v) {
  v += dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f64<0x141>(v);   // row_half_mirror
  return v;
}

// LDS-resident Jacobi: each group of LPP lanes (16) owns one row pair per step, so a wave handles
// 64/LPP pairs with one instruction stream and up to 64 pairs (l <= 128) take 1024 threads.
// EPL = elements of a row per lane = ceil(l / LPP).
// Pair schedule of a sweep (every pair of rows met exactly once): the index range is halved
// recursively.  At a level, every segment [base, base + n) is cut into a top half of h = ceil(n/2) rows
// and a bottom half; in step s top row i meets bottom row (i + s) mod h, so h steps pair every top with
// every bottom of the segment; the next level does the same inside both halves, all segments side by
// side (l-1 .. l+1 steps in all).  Within a level a group keeps its top row in registers and only the
// bottom rows travel through LDS, which halves the LDS traffic of the round-robin schedule.
constexpr int kJLev = 7;      // levels for l <= 128

template <int EPL, int LPP>
__global__ void __launch_bounds__(64 * LPP)
k_jacobi_lds(const double* __restrict__ R, int ldr, int l, int Lp, double* __restrict__ Wg,
             double* __restrict__ sig, int* __restrict__ info, const int* __restrict__ breakdown_flag,
             double tol, double settled) {
  extern __shared__ double W[];
  __shared__ int rotated;
  __shared__ int order_sh[kMaxL];
  __shared__ short tb_top[kJLev][64], tb_bb[kJLev][64], tb_bs[kJLev][64], tb_hi[kJLev][64];
  __shared__ short seg_base[2][128], seg_size[2][128];
  __shared__ int lev_steps[kJLev];
  constexpr int NT = 64 * LPP;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (breakdown_flag && breakdown_flag[0] != 0) {
    if (tid == 0) { info[0] = 0; info[1] = 0; }
    return;
  }
  const int ld = l;
  for (int idx = tid; idx < l * l; idx += NT) {
    int i = idx / l, c = idx - i * l;
    W[i * ld + c] = R[(int64_t)i * ldr + c];
  }
  // schedule tables: per level and group, the top row, the bottom half [bb, bb + bs) and (h << 8) | i
  if (tid == 0) { seg_base[0][0] = 0; seg_size[0][0] = (short)l; }
  for (int lev = 0; lev < kJLev; ++lev) {
    const int nseg = 1 << lev, cur = lev & 1;
    if (tid < 64) tb_top[lev][tid] = -1;
    __syncthreads();
    if (tid < nseg) {
      const int base = seg_base[cur][tid], size = seg_size[cur][tid];
      const int h = (size + 1) >> 1, nb = size - h;
      if (size >= 2) {
        int off = 0;
        for (int k = 0; k < tid; ++k) { const int sz = seg_size[cur][k]; if (sz >= 2) off += (sz + 1) >> 1; }
        for (int i = 0; i < h; ++i) {
          const int gid = off + i;
          if (gid < 64) {
            tb_top[lev][gid] = (short)(base + i); tb_bb[lev][gid] = (short)(base + h);
            tb_bs[lev][gid] = (short)nb; tb_hi[lev][gid] = (short)((h << 8) | i);
          }
        }
      }
      seg_base[cur ^ 1][2 * tid] = (short)base; seg_size[cur ^ 1][2 * tid] = (short)h;
      seg_base[cur ^ 1][2 * tid + 1] = (short)(base + h); seg_size[cur ^ 1][2 * tid + 1] = (short)nb;
    }
    if (tid == 0) {
      int mx = 0;
      for (int k = 0; k < nseg; ++k) { const int sz = seg_size[cur][k]; if (sz >= 2) mx = max(mx, (sz + 1) >> 1); }
      lev_steps[lev] = mx;
    }
    __syncthreads();
  }
  const int pi = tid / LPP;
  const int rl = tid % LPP;
  const double tol2 = tol * tol, settled2 = settled * settled;
  int sweeps = 0, converged = (l < 2);
  __syncthreads();
  while (!converged && sweeps < kMaxSweeps) {
    if (tid == 0) rotated = 0;
    __syncthreads();
    bool any = false;
    for (int lev = 0; lev < kJLev; ++lev) {
      const int steps = lev_steps[lev];
      if (steps == 0) continue;                        // uniform over the workgroup
      const int top = tb_top[lev][pi], bb = tb_bb[lev][pi], bs = tb_bs[lev][pi];
      const int h = tb_hi[lev][pi] >> 8, i0 = tb_hi[lev][pi] & 255;
      double x[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int col = rl + LPP * e;
        x[e] = (top >= 0 && col < l) ? W[top * ld + col] : 0.0;
      }
      for (int step = 0; step < steps; ++step) {
        int j = i0 + step;
        if (j >= h) j -= h;
        const bool valid = top >= 0 && step < h && j < bs;
        const double* wb = W + (bb + j) * ld;
        double y[EPL], al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int col = rl + LPP * e;
          y[e] = (valid && col < l) ? wb[col] : 0.0;
          al = fma(x[e], x[e], al);
          be = fma(y[e], y[e], be);
          ga = fma(x[e], y[e], ga);
        }
        if (LPP == 16) { al = row16_sum(al); be = row16_sum(be); ga = row16_sum(ga); }
        else { al = row8_sum(al); be = row8_sum(be); ga = row8_sum(ga); }
        double c, s;
        bool big;
        const bool rot = rotation(al, be, ga, tol2, settled2, c, s, big) && valid;
        any |= big && valid;
        if (rot) {
          double* wbw = W + (bb + j) * ld;
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            const int col = rl + LPP * e;
            const double xn = c * x[e] - s * y[e];
            if (col < l) wbw[col] = s * x[e] + c * y[e];
            x[e] = xn;
          }
        }
        __syncthreads();
      }
      if (top >= 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int col = rl + LPP * e;
          if (col < l) W[top * ld + col] = x[e];
        }
      }
      __syncthreads();
    }
    if (any) rotated = 1;
    __syncthreads();
    ++sweeps;
    converged = (rotated == 0);
    __syncthreads();
  }
  publish<NT>(W, ld, l, Lp, Wg, sig, order_sh, tid, lane, wave);
  if (tid == 0) { info[0] = sweeps; info[1] = converged; }
}

// ---- large l: block Jacobi, rows in global memory (L2), blocks of kJB rows ---------------------
// The rows are cut into blocks of kJB = 16.  One sweep = one "diagonal" launch, in which every
// workgroup orthogonalises the pairs inside two blocks (round robin within a block), followed by a
// round robin over block pairs, one launch per round: workgroup p loads blocks (I, J) into LDS and
// rotates all kJB x kJB cross pairs in kJB steps (step s pairs row i of I with row (i + s) mod kJB of
// J; the row of I stays in registers, the rows of J travel through LDS), then writes both blocks
// back.  Every pair of rows is met exactly once per sweep; launches replace grid-wide barriers.
constexpr int kJB = 16;

__global__ void k_jacobi_init(const double* __restrict__ R, int ldr, int l, int Lp, double* __restrict__ W) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= l * l) return;
  int i = idx / l, c = idx - i * l;
  W[(int64_t)i * Lp + c] = R[(int64_t)i * ldr + c];
}

// outer < 0: diagonal launch (workgroup p owns blocks 2p and 2p+1); otherwise round `outer` of the
// round robin over nblk2 (even) blocks.  1024 threads = 16 row pairs, one wave per pair (a wave of 64 lanes per
// pair keeps four waves on every SIMD of the CU, which hides the LDS and cross-lane latencies that a quarter wave per
// pair left exposed: 5.3 -> about 1 us per step at l = 272); EPL = ceil(l / 64).
constexpr int kJBLanes = 64;
constexpr int kJBThreads = kJB * kJBLanes;
template <int EPL>
__global__ void __launch_bounds__(kJBThreads)
k_jacobi_block(double* __restrict__ W, int l, int Lp, int nblk2, int outer, double tol, double settled,
               int* __restrict__ rotated) {
  extern __shared__ double sh[];               // 2 * kJB rows of l doubles: block I, then block J
  const int tid = threadIdx.x, pi = tid / kJBLanes, rl = tid % kJBLanes;
  int I, J;
  if (outer < 0) { I = 2 * blockIdx.x; J = I + 1; }
  else rr_pair(blockIdx.x, outer, nblk2, I, J);
  const int rI = I * kJB, rJ = J * kJB;
  if (rI >= l) return;                                  // uniform over the workgroup
  const int nI = min(kJB, l - rI), nJ = max(0, min(kJB, l - rJ));
  if (outer >= 0 && nJ == 0) return;                    // the padding block of an odd block count
  for (int idx = tid; idx < 2 * kJB * l; idx += kJBThreads) {
    const int rr = idx / l, c = idx - rr * l;
    const bool live = rr < kJB ? rr < nI : rr - kJB < nJ;
    const int grow = rr < kJB ? rI + rr : rJ + rr - kJB;
    sh[idx] = live ? W[(int64_t)grow * Lp + c] : 0.0;
  }
  __syncthreads();
  const double tol2 = tol * tol, settled2 = settled * settled;
  bool any = false;
  if (outer < 0) {
    const int blk = pi >> 3, q = pi & 7, nrows = blk == 0 ? nI : nJ;
    for (int step = 0; step < kJB - 1; ++step) {
      int a, b;
      rr_pair(q, step, kJB, a, b);
      const bool valid = b < nrows;                     // a < b
      double* wa = sh + (blk * kJB + a) * l;
      double* wb = sh + (blk * kJB + b) * l;
      double x[EPL], y[EPL], al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int col = rl + kJBLanes * e;
        const bool in = valid && col < l;
        x[e] = in ? wa[col] : 0.0;
        y[e] = in ? wb[col] : 0.0;
        al = fma(x[e], x[e], al); be = fma(y[e], y[e], be); ga = fma(x[e], y[e], ga);
      }
      al = wave64_sum(al); be = wave64_sum(be); ga = wave64_sum(ga);
      double c, s;
      bool big;
      const bool rot = rotation(al, be, ga, tol2, settled2, c, s, big) && valid;
      any |= big && valid;
      if (rot) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int col = rl + kJBLanes * e;
          if (col < l) { wa[col] = c * x[e] - s * y[e]; wb[col] = s * x[e] + c * y[e]; }
        }
      }
      __syncthreads();
    }
  } else {
    double x[EPL];
    double* wa = sh + pi * l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int col = rl + kJBLanes * e;
      x[e] = (pi < nI && col < l) ? wa[col] : 0.0;
    }
    for (int step = 0; step < kJB; ++step) {
      const int j = (pi + step) & (kJB - 1);
      const bool valid = pi < nI && j < nJ;
      double* wb = sh + (kJB + j) * l;
      double y[EPL], al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int col = rl + kJBLanes * e;
        y[e] = (valid && col < l) ? wb[col] : 0.0;
        al = fma(x[e], x[e], al); be = fma(y[e], y[e], be); ga = fma(x[e], y[e], ga);
      }
      al = wave64_sum(al); be = wave64_sum(be); ga = wave64_sum(ga);
      double c, s;
      bool big;
      const bool rot = rotation(al, be, ga, tol2, settled2, c, s, big) && valid;
      any |= big && valid;
      if (rot) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int col = rl + kJBLanes * e;
          const double xn = c * x[e] - s * y[e];
          if (col < l) wb[col] = s * x[e] + c * y[e];
          x[e] = xn;
        }
      }
      __syncthreads();
    }
    if (pi < nI) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int col = rl + kJBLanes * e;
        if (col < l) wa[col] = x[e];
      }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < 2 * kJB * l; idx += kJBThreads) {
    const int rr = idx / l, c = idx - rr * l;
    const bool live = rr < kJB ? rr < nI : rr - kJB < nJ;
    const int grow = rr < kJB ? rI + rr : rJ + rr - kJB;
    if (live) W[(int64_t)grow * Lp + c] = sh[idx];
  }
  if (any && rl == 0) *rotated = 1;
}

__global__ void k_set_int(int* p, int v) { *p = v; }

__global__ void __launch_bounds__(kSvdThreads)
k_jacobi_publish(double* __restrict__ W, int l, int Lp, double* __restrict__ sig, int* __restrict__ info,
                 int sweeps, int converged) {
  __shared__ int order_sh[kMaxL];
  const int tid = threadIdx.x;
  publish<kSvdThreads>(W, Lp, l, Lp, W, sig, order_sh, tid, tid & 63, tid >> 6);
  if (tid == 0) { info[0] = sweeps; info[1] = converged; }
}

// Sorted factors.  Vr[t][i] = W[o_i][t] / s_i;  Ur[kk][i] = sum_t R[kk][t] Vr[t][i] / s_i.
// XV / XU: fp32 zero-padded Lp x Lp right operands of the lifts; Ur / Vr: optional dense fp64.
template <typename TO>
__global__ void k_svd_outputs(const double* __restrict__ R, int ldr, const double* __restrict__ W,
                              const double* __restrict__ sig, int l, int Lp, double* __restrict__ S,
                              TO* __restrict__ S32, TO* __restrict__ XV, TO* __restrict__ XU,
                              double* __restrict__ Ur, double* __restrict__ Vr,
                              const int* __restrict__ breakdown_flag) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= Lp * Lp) return;
  if (breakdown_flag && breakdown_flag[0] != 0) return;   // nothing was computed
  int kk = idx / Lp, i = idx - kk * Lp;
  TO xv = TO(0), xu = TO(0);
  if (kk < l && i < l) {
    const int o = min(max((int)sig[2 * Lp + i], 0), l - 1);   // stays in range even for NaN input
    const double s = sig[i];
    const double* wrow = W + (int64_t)o * Lp;
    double v = 0.0, u = 0.0;
    if (s > 0.0) {
      v = wrow[kk] / s;
      const double* rrow = R + (int64_t)kk * ldr;
      double acc = 0.0;
#pragma unroll 8
      for (int t = 0; t < l; ++t) acc = fma(rrow[t], wrow[t], acc);
      u = acc / (s * s);
    }
    xv = (TO)v; xu = (TO)u;
    if (Vr) Vr[(int64_t)kk * l + i] = v;
    if (Ur) Ur[(int64_t)kk * l + i] = u;
    if (kk == 0) {
      if (S) S[i] = s;
      if (S32) S32[i] = (TO)s;
    }
  }
  if (XV) XV[idx] = xv;
  if (XU) XU[idx] = xu;
}

template <int EPL, int LPP>
static int launch_jacobi_lds(const double* R, int ldr, int l, int Lp, SvdWork& w, const int* breakdown_flag,
                             double tol, double settled, hipStream_t stream) {
  auto kern = k_jacobi_lds<EPL, LPP>;
  const size_t lds = (size_t)l * l * sizeof(double);
  static bool attr_set = false;
  if (!attr_set) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      kJacobiLdsMaxL * kJacobiLdsMaxL * (int)sizeof(double)));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(1), dim3(64 * LPP), lds, stream, R, ldr, l, Lp, w.W, w.sig, w.info,
                     breakdown_flag, tol, settled);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <int EPL>
static int launch_jacobi_block_inst(double* W, int l, int Lp, int nblk2, int outer, double tol, double settled,
                                    int* rotated, hipStream_t stream) {
  auto kern = k_jacobi_block<EPL>;
  static bool attr_set = false;
  if (!attr_set) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      2 * kJB * kMaxL * (int)sizeof(double)));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(nblk2 / 2), dim3(kJBThreads), (size_t)2 * kJB * l * sizeof(double), stream, W, l, Lp, nblk2,
                     outer, tol, settled, rotated);
  return BRSVD_OK;
}
static int launch_jacobi_block(double* W, int l, int Lp, int nblk2, int outer, double tol, double settled, int* rotated,
                               hipStream_t stream) {
  if (l <= 192) return launch_jacobi_block_inst<3>(W, l, Lp, nblk2, outer, tol, settled, rotated, stream);
  if (l <= 320) return launch_jacobi_block_inst<5>(W, l, Lp, nblk2, outer, tol, settled, rotated, stream);
  return launch_jacobi_block_inst<8>(W, l, Lp, nblk2, outer, tol, settled, rotated, stream);
}

template <typename TO>
int small_svd(const double* R, int ldr, int l, int Lp, SvdWork& w, const int* breakdown_flag, double* S,
              TO* S32, TO* XV, TO* XU, double* Ur, double* Vr, hipStream_t stream) {
  if (l < 1 || l > kMaxL) return BRSVD_ERR_ARG;
  const double tol = 1e-13;
  // fp64 factors or singular values asked for: the strict bar; single-precision results only: the relaxed one
  const double settled = (sizeof(TO) == 4 && !S && !Ur && !Vr) ? kSettledF32 : kSettled;
  if (l <= kJacobiLdsMaxL) {
    // Lanes per pair: 16 for l <= 96; above that 8 (fewer, longer instruction streams: the per-pair
    // rotation arithmetic and reductions are issued half as often; 0.88 against 0.92 ms at l = 110).
    if (l <= 32) BRSVD_TRY((launch_jacobi_lds<2, 16>(R, ldr, l, Lp, w, breakdown_flag, tol, settled, stream)));
    else if (l <= 64) BRSVD_TRY((launch_jacobi_lds<4, 16>(R, ldr, l, Lp, w, breakdown_flag, tol, settled, stream)));
    else if (l <= 96) BRSVD_TRY((launch_jacobi_lds<6, 16>(R, ldr, l, Lp, w, breakdown_flag, tol, settled, stream)));
    else if (l <= 112) BRSVD_TRY((launch_jacobi_lds<14, 8>(R, ldr, l, Lp, w, breakdown_flag, tol, settled, stream)));
    else BRSVD_TRY((launch_jacobi_lds<16, 8>(R, ldr, l, Lp, w, breakdown_flag, tol, settled, stream)));
  } else {
    // Host-driven sweeps: the convergence flag is read back once per sweep.
    int* rotated = w.info + 2;
    int host_flag = 0;
    if (breakdown_flag) {
      BRSVD_HIP_TRY(hipMemcpyAsync(&host_flag, breakdown_flag, sizeof(int), hipMemcpyDeviceToHost, stream));
      BRSVD_HIP_TRY(hipStreamSynchronize(stream));
    }
    int sweeps = 0, converged = 0;
    if (host_flag == 0) {
      hipLaunchKernelGGL(k_jacobi_init, dim3((unsigned)ceil_div((int64_t)l * l, 256)), dim3(256), 0, stream, R,
                         ldr, l, Lp, w.W);
      const int nblk = (int)ceil_div(l, kJB), nblk2 = (nblk + 1) & ~1;
      while (!converged && sweeps < kMaxSweeps) {
        hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, stream, rotated, 0);
        for (int outer = -1; outer < nblk2 - 1; ++outer)
          BRSVD_TRY(launch_jacobi_block(w.W, l, Lp, nblk2, outer, tol, settled, rotated, stream));
        BRSVD_HIP_TRY(hipGetLastError());
        int rot = 1;
        BRSVD_HIP_TRY(hipMemcpyAsync(&rot, rotated, sizeof(int), hipMemcpyDeviceToHost, stream));
        BRSVD_HIP_TRY(hipStreamSynchronize(stream));
        ++sweeps;
        converged = (rot == 0);
      }
    }
    if (host_flag == 0)
      hipLaunchKernelGGL(k_jacobi_publish, dim3(1), dim3(kSvdThreads), 0, stream, w.W, l, Lp, w.sig, w.info,
                         sweeps, converged);
    BRSVD_HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(k_svd_outputs<TO>, dim3((unsigned)ceil_div((int64_t)Lp * Lp, 256)), dim3(256), 0, stream, R, ldr,
                     w.W, w.sig, l, Lp, S, S32, XV, XU, Ur, Vr, breakdown_flag);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template int small_svd<float>(const double*, int, int, int, SvdWork&, const int*, double*, float*, float*, float*,
                              double*, double*, hipStream_t);
template int small_svd<double>(const double*, int, int, int, SvdWork&, const int*, double*, double*, double*, double*,
                               double*, double*, hipStream_t);

}  // namespace brsvd
