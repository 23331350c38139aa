// Orthonormalisation of tall thin panels (Alg. 1 step 3, Alg. 2 line 6) on gfx950.
//
// Main route: CholeskyQR applied twice.  G = P^T P is accumulated in fp64 (products of fp32
// values are exact in fp64), factored G = R^T R in fp64, and P <- P * R^-1 is one more thin
// GEMM on the MFMA path.  Pivots that fall below a relative threshold are clamped in every sweep
// but the last one of an output basis; there such a pivot raises the breakdown flag and the caller
// switches to the Householder-based TSQR route (tsqr.hip).
// The paper orthonormalises with a TSQR-based CAQR; range(P) -- all the method needs -- is the
// same for any orthonormalisation.
#include <algorithm>

#include "common.h"

namespace brsvd {

// ---- Gram matrix -----------------------------------------------------------------------------
// G = P^T P on the fp64 matrix cores (v_mfma_f64_16x16x4_f64; products of fp32 values are exact in
// fp64; the panel may also be fp64).  G is cut into blocks of TB x TB tiles of 16 x 16; grid = (row chunks, pairs bi <= bj of
// blocks).  For a step of four panel rows, lane (r, g) of a wave holds P[row + g][16*tile + r] for
// each tile of the two blocks: that value is at once the A operand (entry [i = r][k = g] of the
// transposed tile) and the B operand ([k = g][j = r]), so the panel goes from global memory straight
// into the MFMA operands.  The eight waves of a workgroup take the steps of the chunk round-robin and
// add their accumulators through LDS in wave order; chunks are added by the caller in chunk order.
// Accumulator layout of the instruction: component v of lane (r, g) is entry [g + 4*v][r].
constexpr int kGramWaves = 8;
constexpr int kGramRowStep = 4 * kGramWaves;

__device__ __forceinline__ doublex4 mfma_f64(double a, double b, doublex4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

template <typename T, int TB>
__global__ void __launch_bounds__(kGramWaves * 64)
k_gram(const T* __restrict__ P, int64_t rows, int Lp, int64_t rows_per_chunk, double* __restrict__ Gpart) {
  __shared__ double red[kGramWaves][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 15, g = lane >> 4;
  const int NT = Lp / 16, nb = (NT + TB - 1) / TB;
  int bi = 0, rem = blockIdx.y;
  while (rem >= nb - bi) { rem -= nb - bi; ++bi; }
  const int bj = bi + rem;
  const int ti_n = min(TB, NT - bi * TB), tj_n = min(TB, NT - bj * TB);
  const bool diag = bi == bj;
  const int64_t rbeg = (int64_t)blockIdx.x * rows_per_chunk;
  const int64_t rend = min(rows, rbeg + rows_per_chunk);
  const T* pi = P + 16 * (bi * TB) + r;
  const T* pj = P + 16 * (bj * TB) + r;

  doublex4 acc[TB][TB];
#pragma unroll
  for (int i = 0; i < TB; ++i)
#pragma unroll
    for (int j = 0; j < TB; ++j) acc[i][j] = doublex4{0.0, 0.0, 0.0, 0.0};

  T an[TB], bn[TB];
  auto load = [&](int64_t row0) {
    const int64_t row = row0 + g;
    const bool valid = row < rend;
    const int64_t off = (valid ? row : rbeg) * Lp;
#pragma unroll
    for (int t = 0; t < TB; ++t) {
      an[t] = (valid && t < ti_n) ? pi[off + 16 * t] : T(0);
      bn[t] = (valid && t < tj_n && !diag) ? pj[off + 16 * t] : T(0);
    }
  };
  int64_t row0 = rbeg + 4 * wave;
  if (row0 < rend) load(row0);
  for (; row0 < rend; row0 += kGramRowStep) {
    double a[TB], b[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) { a[t] = (double)an[t]; b[t] = diag ? a[t] : (double)bn[t]; }
    if (row0 + kGramRowStep < rend) load(row0 + kGramRowStep);     // next step's rows, in flight under the MFMAs
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
      for (int j = 0; j < TB; ++j)
        if (i < ti_n && j < tj_n && !(diag && j < i)) acc[i][j] = mfma_f64(a[i], b[j], acc[i][j]);
  }

  double* Go = Gpart + (int64_t)blockIdx.x * Lp * Lp;
#pragma unroll
  for (int i = 0; i < TB; ++i)
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      if (!(i < ti_n && j < tj_n && !(diag && j < i))) continue;      // uniform over the workgroup
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][v * 64 + lane] = acc[i][j][v];
      __syncthreads();
      if (tid < 256) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kGramWaves; ++w) s += red[w][tid];
        const int v = tid >> 6, ln = tid & 63;
        const int gi = 16 * (bi * TB + i) + (ln >> 4) + 4 * v, gj = 16 * (bj * TB + j) + (ln & 15);
        Go[(int64_t)gi * Lp + gj] = s;
      }
      __syncthreads();
    }
}

// ---- Cholesky factor and its inverse ---------------------------------------------------------
// One workgroup of 1024 threads; blocked right-looking factorisation G = R^T R with 16 x 16
// blocks, then R^-1 by recursive doubling (invert the diagonal blocks, then merge neighbouring
// blocks: inv([R11 R12; 0 R22]) = [X11, -X11 R12 X22; 0, X22]).  Everything is fp64.  For
// Lp <= kCholLdsMaxLp the matrix lives in LDS for the whole kernel; above that it stays in global
// memory (L2) and only the current 16-row panel is mirrored in LDS.
// A pivot <= tol * its original diagonal entry is clamped to that value (lenient) or sets
// flag[0] = 1 + column and ends the kernel.
constexpr int kNB = 16;
constexpr int kCholLdsMaxLp = 128;    // largest padded size whose (Lp x (Lp+1)) fp64 matrix fits the LDS

// Broadcast of lane `src` (a compile-time constant after unrolling): two scalar lane reads.
__device__ __forceinline__ double shfl_d(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}
// 1/sqrt(x) and 1/x: hardware seed plus two Newton steps (full fp64 accuracy for normal x).
__device__ __forceinline__ double rsqrt_fast(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double h = 0.5 * x;
  y = fma(y, fma(-h * y, y, 0.5), y);
  y = fma(y, fma(-h * y, y, 0.5), y);
  return y;
}
__device__ __forceinline__ double rcp_fast(double x) {
  double y = __builtin_amdgcn_rcp(x);
  y = fma(y, fma(-x, y, 1.0), y);
  y = fma(y, fma(-x, y, 1.0), y);
  return y;
}

// Wave-level Cholesky of the 16 x 16 diagonal block at (kb, kb).  The tile sits in the MFMA
// accumulator layout (lane (r, g), component v = entry [g + 4 v][r]), so that the four rows 4p .. 4p+3 of
// a panel are one register across the wave.  Per panel: the four rows are gathered into every lane
// (lane r keeps column r of them), factored in four pivot steps with lane broadcasts, and the rest of
// the tile receives their rank-4 update as a single v_mfma_f64_16x16x4_f64 with the panel as both
// operands.  Pivots at or below tol * (original diagonal) are clamped (see k_chol_inv); returns false
// if that happened.  Writes R_kk into M (upper part) and into Rkk (16 x 17, spare column = 1/diagonal).
__device__ bool chol_diag_wave(double* M, int64_t ld, int kb, int nb, const double* d0, double tol,
                               double* Rkk, int lane) {
  (void)nb;
  const int r = lane & 15, g = lane >> 4;
  doublex4 t;
#pragma unroll
  for (int v = 0; v < 4; ++v) t[v] = M[(int64_t)(kb + g + 4 * v) * ld + kb + r];
  bool ok = true;
#pragma unroll
  for (int p4 = 0; p4 < 4; ++p4) {
    const int jb = 4 * p4;
    double pr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double x = __shfl(t[p4], 16 * i + r, 64);           // entry [jb + i][r]
      pr[i] = r >= jb + i ? x : 0.0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = jb + i;
      double d = shfl_d(pr[i], j);
      const double floor_ = tol * d0[kb + j];
      if (!(d > floor_)) { ok = false; d = floor_ > 0.0 ? floor_ : 1.0; }   // an all-zero column keeps R_jj = 1
      const double inv = rsqrt_fast(d);
      const double ri = r > j ? pr[i] * inv : (r == j ? d * inv : 0.0);
      pr[i] = ri;
#pragma unroll
      for (int i2 = i + 1; i2 < 4; ++i2) {
        const double s = shfl_d(ri, jb + i2);
        if (r >= jb + i2) pr[i2] -= s * ri;
      }
    }
    const double rowv = g == 0 ? pr[0] : (g == 1 ? pr[1] : (g == 2 ? pr[2] : pr[3]));   // row jb + g, column r
    if (r >= jb + g) M[(int64_t)(kb + jb + g) * ld + kb + r] = rowv;
    Rkk[(jb + g) * 17 + r] = rowv;
    if (r == jb + g) Rkk[(jb + g) * 17 + 16] = rcp_fast(rowv);    // 1 / R[j][j] in the spare column, for the panel solve
    if (p4 < 3) t = mfma_f64(-rowv, rowv, t);
  }
  return ok;
}

// In-place inverse of the nb x nb upper-triangular diagonal block at (kb, kb), one wave.
__device__ void inv_diag_wave(double* M, int ld, int kb, int nb, int lane) {
  const int c = lane & 15;
  double rc[kNB], x[kNB];
#pragma unroll
  for (int i = 0; i < kNB; ++i) {
    rc[i] = (i < nb && c < nb) ? (i <= c ? M[(int64_t)(kb + i) * ld + kb + c] : 0.0) : (i == c ? 1.0 : 0.0);
    x[i] = 0.0;
  }
  // x = column c of the inverse: x[c] = 1/r[c][c]; x[i] = -(sum_{t=i+1..c} r[i][t] x[t]) / r[i][i]
#pragma unroll
  for (int i = kNB - 1; i >= 0; --i) {
    double s = 0.0;
#pragma unroll
    for (int t = i + 1; t < kNB; ++t) {
      const double rit = shfl_d(rc[i], t);      // r[i][t] lives in lane t
      if (t <= c) s = fma(rit, x[t], s);
    }
    const double inv_rii = rcp_fast(shfl_d(rc[i], i));
    if (i == c) x[i] = inv_rii;
    else if (i < c) x[i] = -s * inv_rii;
  }
  if (lane < kNB && c < nb) {
#pragma unroll
    for (int i = 0; i < kNB; ++i)
      if (i <= c) M[(int64_t)(kb + i) * ld + kb + c] = x[i];
  }
}

// Trailing update of one 16 x 16 tile on the fp64 matrix cores: M[r0.., c0..] -= P[:, r0..]^T P[:, c0..],
// P = the 16 freshly solved rows of R (row stride ldp).  Lane (r, g) holds P[4*kk + g][. + r] as A and
// B operand of step kk; accumulator component v of lane (r, g) is entry [g + 4*v][r].
__device__ __forceinline__ void trailing_tile(double* M, int64_t ld, const double* P, int ldp, int r0, int c0,
                                              int lane) {
  const int r = lane & 15, g = lane >> 4;
  double* mt = M + (int64_t)(r0 + g) * ld + c0 + r;
  doublex4 acc;
#pragma unroll
  for (int v = 0; v < 4; ++v) acc[v] = mt[(int64_t)4 * v * ld];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const double* prow = P + (4 * kk + g) * ldp;
    acc = mfma_f64(-prow[r0 + r], prow[c0 + r], acc);
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) mt[(int64_t)4 * v * ld] = acc[v];
}

// The working matrix is padded to Lp x Lp with an identity block, so that every block is a full
// 16 x 16 tile.  Schedule of the factorisation: wave 0 factors the diagonal block of step k+1 (after
// updating that one tile) while the other waves finish the trailing update of step k, which takes
// the 16-step pivot chain off the critical path of all but the first block.
template <bool IN_LDS, typename TO>
__global__ void __launch_bounds__(1024)
k_chol_inv(double* __restrict__ G, int l, int Lp, double* __restrict__ Rout, double* __restrict__ Xtmp,
           TO* __restrict__ Rinv_out, int* __restrict__ flag, double tol, int factored, int lenient) {
  extern __shared__ double smem[];
  __shared__ int bad;
  double* Rkk = smem;                 // 16 x 17
  double* d0 = smem + 16 * 17;        // kMaxL
  double* rest = d0 + kMaxL;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (flag[0] != 0) return;           // an earlier panel already broke down: results are void anyway
  double* M;
  int ld;
  double* pan;                        // current 16-row panel R[kb:kb+16, :] (row stride ldp)
  int ldp;
  if (IN_LDS) {
    M = rest; ld = Lp + 1;
    for (int idx = tid; idx < Lp * Lp; idx += 1024) {
      const int i = idx / Lp, c = idx - i * Lp;
      M[i * ld + c] = (i < l && c < l) ? (c >= i ? G[(int64_t)i * Lp + c] : 0.0) : (i == c ? 1.0 : 0.0);
    }
    pan = nullptr; ldp = ld;
  } else {
    M = G; ld = Lp;
    for (int idx = tid; idx < Lp * Lp; idx += 1024) {
      const int i = idx / Lp, c = idx - i * Lp;
      if (i >= l || c >= l) M[(int64_t)i * ld + c] = i == c ? 1.0 : 0.0;
    }
    pan = rest; ldp = kMaxL;
  }
  if (tid == 0) bad = 0;
  __syncthreads();
  for (int i = tid; i < Lp; i += 1024) d0[i] = M[(int64_t)i * ld + i];
  __syncthreads();

  // ---- factorisation (skipped when G already holds an upper-triangular factor) ----
  if (!factored) {
    if (wave == 0) {
      const bool ok = chol_diag_wave(M, ld, 0, kNB, d0, tol, Rkk, lane);
      if (!ok && !lenient && lane == 0) bad = 1;
    }
    __syncthreads();
    if (bad) {
      if (tid == 0) flag[0] = bad;
      return;
    }
  }
  for (int kb = factored ? Lp : 0; kb < Lp; kb += kNB) {
    const int t0 = kb + kNB;          // first trailing column
    // row panel: R[kb:kb+16, c] = R_kk^-T G[kb:kb+16, c], one column per thread
    for (int c = t0 + tid; c < Lp; c += 1024) {
      double x[kNB];
#pragma unroll
      for (int i = 0; i < kNB; ++i) {
        double sacc = M[(int64_t)(kb + i) * ld + c];
#pragma unroll
        for (int t = 0; t < kNB; ++t)
          if (t < i) sacc = fma(-Rkk[t * 17 + i], x[t], sacc);
        x[i] = sacc * Rkk[i * 17 + 16];
        M[(int64_t)(kb + i) * ld + c] = x[i];
        if (!IN_LDS) pan[i * ldp + c] = x[i];
      }
    }
    __syncthreads();
    // trailing update, upper tiles (ti <= tj) of the (Lp - t0)^2 block; tile 0 = (0, 0) is the next
    // diagonal block: wave 0 updates it and factors it at once, waves 1..15 share the other tiles
    const double* P = IN_LDS ? (M + (int64_t)kb * ld) : pan;
    const int T16 = (Lp - t0) / kNB;
    const int ntile = T16 * (T16 + 1) / 2;
    if (wave == 0) {
      if (ntile > 0) {
        trailing_tile(M, ld, P, ldp, t0, t0, lane);
        const bool ok = chol_diag_wave(M, ld, t0, kNB, d0, tol, Rkk, lane);
        if (!ok && !lenient && lane == 0) bad = t0 + 1;
      }
    } else {
      for (int idx = wave; idx < ntile; idx += 15) {
        int ti = 0, rem = idx;
        while (rem >= T16 - ti) { rem -= T16 - ti; ++ti; }
        trailing_tile(M, ld, P, ldp, t0 + kNB * ti, t0 + kNB * (ti + rem), lane);
      }
    }
    __syncthreads();
    if (bad) {
      if (tid == 0) flag[0] = bad;
      return;
    }
  }

  // ---- publish R ----
  if (Rout) {
    for (int idx = tid; idx < l * l; idx += 1024) {
      int i = idx / l, c = idx - i * l;
      Rout[(int64_t)i * Lp + c] = c >= i ? M[(int64_t)i * ld + c] : 0.0;
    }
  }
  __syncthreads();

  // ---- inverse, level 0: diagonal blocks, one wave each (the padding block is an identity) ----
  const int nblk = Lp / kNB;
  for (int bi = wave; bi < nblk; bi += 16) inv_diag_wave(M, ld, bi * kNB, kNB, lane);
  __syncthreads();
  // ---- merge levels on the fp64 matrix cores: X12 = -X11 (R12 X22), tile by tile.  A pair at level B
  // (in tiles) joins the inverted blocks [a0, a0+B) and [a0+B, a0+B+w).  Phase 0 forms T = R12 X22
  // (X22 upper triangular: tiles tk <= tj), phase 1 forms X12 = -X11 T (tiles tk >= ti).  Diagonal tiles
  // of X11 / X22 are masked to their upper triangle (their lower part holds leftovers of the trailing
  // updates).  LDS variant: at most 16 tiles per phase, one per wave, held in registers until every
  // wave has finished reading, then written in place.  Global variant: T goes to the scratch Xtmp. ----
  {
    const int r = lane & 15, g = lane >> 4;
    for (int B = 1; B < nblk; B *= 2) {
      const int npair = (nblk + 2 * B - 1) / (2 * B);
      for (int phase = 0; phase < 2; ++phase) {
        doublex4 keep = {0.0, 0.0, 0.0, 0.0};
        int kr0 = -1, kc0 = 0;
        int tile = 0;                                   // running tile index over all pairs of this level
        for (int p = 0; p < npair; ++p) {
          const int a0 = 2 * B * p;                     // in tiles
          const int w = min(a0 + 2 * B, nblk) - (a0 + B);
          if (w <= 0) continue;
          for (int t = 0; t < B * w; ++t, ++tile) {
            if ((tile & 15) != wave) continue;
            const int ti = t / w, tj = t - ti * w;      // tile row within the left block, tile column within the right
            const int r0 = (a0 + ti) * kNB, c0 = (a0 + B + tj) * kNB;
            doublex4 acc = {0.0, 0.0, 0.0, 0.0};
            if (phase == 0) {
              for (int tk = 0; tk <= tj; ++tk) {
                const int k0 = (a0 + B + tk) * kNB;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                  const int k = 4 * kk + g;
                  const double av = M[(int64_t)(r0 + r) * ld + k0 + k];                       // R12[i = r][k]
                  double bv = M[(int64_t)(k0 + k) * ld + c0 + r];                             // X22[k][j = r]
                  if (tk == tj && k > r) bv = 0.0;
                  acc = mfma_f64(av, bv, acc);
                }
              }
            } else {
              const double* Tm = IN_LDS ? M : Xtmp;
              const int64_t ldt = IN_LDS ? ld : Lp;
              for (int tk = ti; tk < B; ++tk) {
                const int k0 = (a0 + tk) * kNB;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                  const int k = 4 * kk + g;
                  double av = M[(int64_t)(r0 + r) * ld + k0 + k];                             // X11[i = r][k]
                  if (tk == ti && r > k) av = 0.0;
                  const double bv = Tm[(int64_t)(k0 + k) * ldt + c0 + r];                     // T[k][j = r]
                  acc = mfma_f64(-av, bv, acc);
                }
              }
            }
            // accumulator component v of lane (r, g) is entry [g + 4 v][r] of the tile
            if (IN_LDS) {
              keep = acc; kr0 = r0; kc0 = c0;
            } else {
              double* dst = phase == 0 ? Xtmp : M;
              const int64_t ldd = phase == 0 ? Lp : ld;
#pragma unroll
              for (int v = 0; v < 4; ++v) dst[(int64_t)(r0 + g + 4 * v) * ldd + c0 + r] = acc[v];
            }
          }
        }
        __syncthreads();
        if (IN_LDS && kr0 >= 0) {
#pragma unroll
          for (int v = 0; v < 4; ++v) M[(int64_t)(kr0 + g + 4 * v) * ld + kc0 + r] = keep[v];
        }
        __syncthreads();
      }
    }
  }
  // R^-1 in the panels' type, zero below the diagonal and in the padding
  for (int idx = tid; idx < Lp * Lp; idx += 1024) {
    const int i = idx / Lp, c = idx - i * Lp;
    Rinv_out[idx] = (i < l && c < l && c >= i) ? (TO)M[(int64_t)i * ld + c] : TO(0);
  }
}

// Rtot = R2 * R1 (both upper triangular, l x l, stride Lp).
__global__ void k_triu_mul(const double* __restrict__ R2, const double* __restrict__ R1, int l, int Lp,
                           double* __restrict__ Rtot) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= l * l) return;
  int i = idx / l, c = idx - i * l;
  double s = 0.0;
#pragma unroll 8
  for (int k = i; k <= c; ++k) s = fma(R2[(int64_t)i * Lp + k], R1[(int64_t)k * Lp + c], s);
  Rtot[(int64_t)i * Lp + c] = s;
}

// Row chunks of the Gram kernel.  Up to 64 chunks of at least 64 rows fill the chip for panels of
// ordinary height; very tall panels get one chunk per 1024 rows, bounded by about 2048 workgroups
// per launch and 64 MB of partial sums.  The partial sums are added in chunk order (in two levels
// of at most kGramFan terms when there are more than kGramFan chunks), so the result is deterministic.
constexpr int kGramFan = 64;
uint64_t orth_gram_chunks(int64_t rows, int Lp) {
  const int nbk = (Lp + 63) / 64, pairs = nbk * (nbk + 1) / 2;
  int64_t c = std::min<int64_t>(ceil_div(rows, 64), 64);
  c = std::min<int64_t>(c, std::max<int64_t>(1, ceil_div(1024, pairs)));
  const int64_t cap = std::min<int64_t>(std::max(2048 / pairs, 1), (64ll << 20) / ((int64_t)Lp * Lp * 8));
  const int64_t tall = std::min<int64_t>(rows / 1024, cap);
  return (uint64_t)std::max<int64_t>(std::max(c, tall), 1);
}
// Slots of Lp x Lp doubles the partial sums need (chunks, plus the first-level sums).
uint64_t orth_gram_slots(int64_t rows, int Lp) {
  const uint64_t c = orth_gram_chunks(rows, Lp);
  return c > (uint64_t)kGramFan ? c + ceil_div(c, kGramFan) : c;
}

// out[g] = sum of the slots [g*fan, min((g+1)*fan, nsplit)) of part, in slot order.
__global__ void k_reduce_groups(const double* __restrict__ part, int nsplit, int fan, int64_t count,
                                double* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= count) return;
  const int s0 = blockIdx.y * fan, s1 = min(nsplit, s0 + fan);
  double s = 0.0;
#pragma unroll 8
  for (int i = s0; i < s1; ++i) s += part[(int64_t)i * count + idx];
  out[(int64_t)blockIdx.y * count + idx] = s;
}

template <typename T>
static int gram(const T* P, int64_t rows, int Lp, OrthWorkT<T>& w, hipStream_t stream) {
  int chunks = (int)orth_gram_chunks(rows, Lp);
  if ((int64_t)orth_gram_slots(rows, Lp) > w.gram_chunks_max) return BRSVD_ERR_BUDGET;
  int64_t rpc = ceil_div(rows, chunks);
  rpc = ceil_div(rpc, kGramRowStep) * kGramRowStep;
  chunks = (int)ceil_div(rows, rpc);
  const int nt = Lp / 16, nb = (nt + 3) / 4;       // blocks of (up to) four tiles; a single smaller block when nt < 4
  dim3 grid(chunks, nb * (nb + 1) / 2), block(kGramWaves * 64);
  switch (nt) {
    case 1: hipLaunchKernelGGL((k_gram<T, 1>), grid, block, 0, stream, P, rows, Lp, rpc, w.gram_part); break;
    case 2: hipLaunchKernelGGL((k_gram<T, 2>), grid, block, 0, stream, P, rows, Lp, rpc, w.gram_part); break;
    case 3: hipLaunchKernelGGL((k_gram<T, 3>), grid, block, 0, stream, P, rows, Lp, rpc, w.gram_part); break;
    default: hipLaunchKernelGGL((k_gram<T, 4>), grid, block, 0, stream, P, rows, Lp, rpc, w.gram_part); break;
  }
  BRSVD_HIP_TRY(hipGetLastError());
  const int64_t count = (int64_t)Lp * Lp;
  const unsigned bx = (unsigned)ceil_div(count, 256);
  // small factors (up to 64 x 64) are summed in one level up to 256 chunks: a thread's serial sum is short against a
  // second launch on the latency-bound chain Gram -> Cholesky -> apply
  const int fan = count <= 4096 ? 4 * kGramFan : kGramFan;
  if (chunks > fan) {
    const int groups = (int)ceil_div(chunks, kGramFan);
    double* lvl1 = w.gram_part + (int64_t)chunks * count;
    hipLaunchKernelGGL(k_reduce_groups, dim3(bx, groups), dim3(256), 0, stream, w.gram_part, chunks, kGramFan, count,
                       lvl1);
    hipLaunchKernelGGL(k_reduce_groups, dim3(bx, 1), dim3(256), 0, stream, lvl1, groups, groups, count, w.G);
  } else {
    hipLaunchKernelGGL(k_reduce_groups, dim3(bx, 1), dim3(256), 0, stream, w.gram_part, chunks, chunks, count, w.G);
  }
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

// lenient != 0: pivots below tol * (original diagonal) are clamped and the factorisation goes on;
// otherwise such a pivot raises the breakdown flag and ends the kernel.
template <typename TO>
static int chol_inv(double* G, int l, int Lp, double* Rout, double* Xtmp, TO* Rinv, int* flags, double tol,
                    hipStream_t stream, int factored = 0, int lenient = 0) {
  const bool in_lds = Lp <= kCholLdsMaxLp;
  const size_t lds = (16 * 17 + kMaxL + (in_lds ? (size_t)Lp * (Lp + 1) : (size_t)kNB * kMaxL)) * sizeof(double);
  static bool attr_set = false;
  if (!attr_set) {
    const int max_lds = (16 * 17 + kMaxL + kCholLdsMaxLp * (kCholLdsMaxLp + 1)) * (int)sizeof(double);
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)k_chol_inv<true, TO>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      max_lds));
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)k_chol_inv<false, TO>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (16 * 17 + kMaxL + kNB * kMaxL) * (int)sizeof(double)));
    attr_set = true;
  }
  if (in_lds)
    hipLaunchKernelGGL((k_chol_inv<true, TO>), dim3(1), dim3(1024), lds, stream, G, l, Lp, Rout, Xtmp, Rinv, flags, tol,
                       factored, lenient);
  else
    hipLaunchKernelGGL((k_chol_inv<false, TO>), dim3(1), dim3(1024), lds, stream, G, l, Lp, Rout, Xtmp, Rinv, flags,
                       tol, factored, lenient);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T>
int chol_inv_factored(double* G, int l, int Lp, double* Rout, double* Xtmp, T* Rinv, int* flags, hipStream_t stream) {
  return chol_inv<T>(G, l, Lp, Rout, Xtmp, Rinv, flags, 0.0, stream, 1);
}

template <typename T>
int apply_to_companion(OrthWorkT<T>& w, int Lp, hipStream_t stream) {
  if (!w.comp) return BRSVD_OK;
  BRSVD_TRY(gemm_an(w.comp, Lp, w.comp_rows, Lp, w.Rinv, Lp, w.comp_tmp, Lp, Lp, w.gemm_scratch, w.gemm_scratch_bytes,
                    stream));
  T* t = w.comp; w.comp = w.comp_tmp; w.comp_tmp = t;
  return BRSVD_OK;
}

// *out = min_i |R_ii| / max_i |R_ii| of an l x l triangular factor (stride Lp): how far the last column
// of the factored panel sits below the first.  One wave.
__global__ void __launch_bounds__(64)
k_diag_ratio(const double* __restrict__ R, int l, int Lp, double* __restrict__ out) {
  double lo = INFINITY, hi = 0.0;
  for (int i = threadIdx.x; i < l; i += 64) {
    const double d = fabs(R[(int64_t)i * Lp + i]);
    lo = fmin(lo, d);
    hi = fmax(hi, d);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = fmin(lo, __shfl_xor(lo, off, 64));
    hi = fmax(hi, __shfl_xor(hi, off, 64));
  }
  if (threadIdx.x == 0) *out = hi > 0.0 ? lo / hi : 0.0;
}

int diag_ratio(const double* R, int l, int Lp, double* out, hipStream_t stream) {
  hipLaunchKernelGGL(k_diag_ratio, dim3(1), dim3(64), 0, stream, R, l, Lp, out);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

int triu_mul(const double* R2, const double* R1, int l, int Lp, double* Rtot, hipStream_t stream) {
  hipLaunchKernelGGL(k_triu_mul, dim3((unsigned)ceil_div((int64_t)l * l, 256)), dim3(256), 0, stream, R2, R1, l, Lp,
                     Rtot);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

// Only the last sweep of a basis that reaches the output must succeed without clamped pivots (its
// input is then already nearly orthonormal, so a small pivot there means the panel really lost
// rank to working precision).  Earlier sweeps, and the single sweep of an intermediate panel, clamp:
// the numerically dependent directions of an exactly rank-deficient panel -- the paper's own test
// inputs have rank k < l -- come out as damped rounding noise, which the next sweep or the next
// power step treats like any other direction; P = Q R holds exactly either way.
template <typename T>
int cholqr_sweeps(T* P, T* tmp, int64_t rows, int l, int Lp, int nsweeps, OrthWorkT<T>& w, double* Rtot,
                  T** result, hipStream_t stream, bool strict_last, bool publish_R) {
  const double tol = 1e-12;
  T* src = P;
  T* dst = tmp;
  for (int sweep = 0; sweep < nsweeps; ++sweep) {
    BRSVD_TRY(gram<T>(src, rows, Lp, w, stream));
    const int lenient = (sweep + 1 < nsweeps || !strict_last) ? 1 : 0;
    double* Rs = (Rtot || publish_R) ? w.R[sweep] : nullptr;      // the factor is only written out when someone reads it
    BRSVD_TRY(chol_inv<T>(w.G, l, Lp, Rs, w.Xinv, w.Rinv, w.flags, tol, stream, 0, lenient));
    BRSVD_TRY(gemm_an(src, Lp, rows, Lp, w.Rinv, Lp, dst, Lp, Lp, w.gemm_scratch, w.gemm_scratch_bytes, stream));
    BRSVD_TRY(apply_to_companion<T>(w, Lp, stream));
    T* t = src; src = dst; dst = t;
  }
  *result = src;
  if (Rtot) {
    if (nsweeps == 2) {
      BRSVD_TRY(triu_mul(w.R[1], w.R[0], l, Lp, Rtot, stream));
    } else {
      BRSVD_HIP_TRY(hipMemcpyAsync(Rtot, w.R[0], (size_t)Lp * Lp * sizeof(double), hipMemcpyDeviceToDevice, stream));
    }
  }
  return BRSVD_OK;
}

template <typename T>
int orth_panel(T* P, T* tmp, int64_t rows, int l, int Lp, int method, bool final_basis, OrthWorkT<T>& w,
               double* Rtot, T** result, hipStream_t stream) {
  if (rows < l) return BRSVD_ERR_ARG;
  if (method == BRSVD_ORTH_TSQR) return tsqr_panel<T>(P, tmp, rows, l, Lp, w, Rtot, result, stream);
  // A panel that only seeds the next power half step needs a well-conditioned basis, not one
  // orthonormal to working precision: one CholeskyQR sweep (fp64 Gram) leaves ||Q^T Q - I|| of
  // order eps32 * cond(P).  The bases that reach the output (Q behind U, W_B behind V) get two.
  return cholqr_sweeps<T>(P, tmp, rows, l, Lp, final_basis ? 2 : 1, w, Rtot, result, stream, final_basis);
}

#define BRSVD_ORTH_INSTANTIATE(T)                                                                               \
  template int chol_inv_factored<T>(double*, int, int, double*, double*, T*, int*, hipStream_t);                \
  template int apply_to_companion<T>(OrthWorkT<T>&, int, hipStream_t);                                          \
  template int cholqr_sweeps<T>(T*, T*, int64_t, int, int, int, OrthWorkT<T>&, double*, T**, hipStream_t, bool, \
                                bool);                                                                          \
  template int orth_panel<T>(T*, T*, int64_t, int, int, int, bool, OrthWorkT<T>&, double*, T**, hipStream_t);
BRSVD_ORTH_INSTANTIATE(float)
BRSVD_ORTH_INSTANTIATE(double)
#undef BRSVD_ORTH_INSTANTIATE

}  // namespace brsvd
