// Thin-panel GEMMs of the randomized range finder on the matrix cores (gfx950, wave64): fp32 on
// v_mfma_f32_16x16x4_f32 and, from the same templates, fp64 on v_mfma_f64_16x16x4_f64.
//
//   gemm_an:  Y_I = A_I * X        sketch Y = A*Omega and the power step Y = A*W
//                                  (Alg. 1 step 2, Alg. 2 line 4; factors applied right to left,
//                                  Sec. 3 "Implementation details")
//   gemm_at:  Z  += A_I^T * Q_I    power half step Z = A^T*Q and the projection B^T = A^T*Q
//                                  (Alg. 1 step 4, Alg. 2 line 9)
//
// Both read each element of the row block A_I exactly once, straight from HBM into the MFMA
// A-operand registers (no LDS round trip for A), while the thin panel (X or Q) is staged
// through a double-buffered LDS tile shared by the waves of a workgroup.
//
// Operand layout of both instructions (lane = 16*g + r, g = 0..3, r = 0..15):
//   A operand: lane holds a[i = r][k = g];  B operand: lane holds b[k = g][j = r];
//   D: lane holds d[i = 4*g + v][j = r] (fp32) or d[i = g + 4*v][j = r] (fp64) in component v = 0..3.
// Because the contraction index may be visited in any order, a lane's vector of four
// consecutive k (gemm_an) or of MT consecutive columns (gemm_at) feeds that many MFMAs directly.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>

#include "common.h"

namespace brsvd {

__device__ __forceinline__ floatx4 mfma16(float a, float b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ doublex4 mfma16(double a, double b, doublex4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// Per element type: vector of four elements (MFMA accumulator, and four consecutive k of A), the
// 16-byte unit the panel is staged with, and where accumulator component v of lane (r, g) sits in the
// 16 x 16 tile: row 4*g + v for v_mfma_f32_16x16x4_f32, row g + 4*v for v_mfma_f64_16x16x4_f64
// (column r for both).  The fp64 kernels are the same code at half the tile widths.
template <typename T> struct El;
template <> struct El<float> {
  typedef floatx4 v4;
  typedef floatx4 v4u __attribute__((aligned(4)));     // four consecutive elements at any element address
  typedef floatx4 u16;
  static constexpr int kPerU16 = 4;
  static constexpr int kBankMod = 64;      // row strides are padded against 64 banks of 4 bytes
  __device__ static __forceinline__ int acc_row(int g, int v) { return 4 * g + v; }
};
template <> struct El<double> {
  typedef doublex4 v4;
  typedef doublex4 v4u __attribute__((aligned(8)));
  typedef double u16 __attribute__((ext_vector_type(2)));
  static constexpr int kPerU16 = 2;
  static constexpr int kBankMod = 32;
  __device__ static __forceinline__ int acc_row(int g, int v) { return g + 4 * v; }
};

// Streaming (nontemporal) load for the instances whose rows start on 16-byte boundaries, plain load for the
// RAGGED ones: rows at other alignments share their first and last cache lines with the neighbouring accesses,
// and a streaming load does not keep a line for the neighbour.  A macro, so that the pointer keeps the reduced
// alignment of its type (a function template would deduce the fully aligned vector type).
#define BRSVD_LOAD_A(P) (RAGGED ? *(P) : __builtin_nontemporal_load(P))

// Identity the compiler cannot see through: the result is a new value living in VGPRs.  Used to
// hand the prefetched block of A over to the MFMA stream, so that (a) the wait for the prefetch
// sits exactly here and (b) no MFMA operand is mapped onto a register with a load in flight.
template <typename V>
__device__ __forceinline__ V opaque(V v) {
  asm volatile("" : "+v"(v));
  return v;
}

constexpr int kMaxNT = 17;   // n-tiles (of 16 columns) one launch keeps in registers

// --------------------------------------------------------------------------------------------
// gemm_an
// --------------------------------------------------------------------------------------------
// Workgroup: WAVES waves, wave w owns rows [row0 + w*MT*16, +MT*16) of a row tile and all NT*16 columns.
// How a launch is cut into workgroups (AnShape): with S resident workgroup slots on the chip,
//   * the first `whole` row tiles (a multiple of S) get one workgroup each, which runs over the whole
//     contraction and writes Y directly: full rounds of equal work;
//   * the `lt` leftover tiles are cut along the contraction so that they fill one more, shorter round
//     evenly: f main splits per tile (slot s = chunks [s*(C-x)/f, (s+1)*(C-x)/f)) and, for the S - f*lt
//     slots that would otherwise idle, a tail strip [C-x, C) of every leftover tile, j strips per extra
//     workgroup, with x chosen so that j strips weigh as much as one main split.
// Workgroups of one kind walk the contraction in lockstep, so the panel chunks they share stay in L2.
// The partial panels of a leftover tile (slots 0..f-1, then the tail) are added in that order.
struct AnShape {
  int C, whole, lt, f, x, j;
};

template <typename T, int NT, int MT, int WAVES, int KC, bool RAGGED>
__global__ void __launch_bounds__(WAVES * 64)
k_gemm_an(const T* __restrict__ A, int64_t lda, int rows, int K,
          const T* __restrict__ X, int ldx,
          T* __restrict__ Y, int64_t ldy, int ncols,
          T* __restrict__ Part, int64_t ldp, int64_t split_stride, AnShape sh) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  T* lds = reinterpret_cast<T*>(lds_raw);
  typedef typename El<T>::v4 vec4;
  typedef typename El<T>::v4u vec4u;
  typedef typename El<T>::u16 unit16;
  constexpr int EPU = El<T>::kPerU16;
  constexpr int NTHREADS = WAVES * 64;
  constexpr int LD = NT * 16 + 4;          // +4: the four k-groups of a wave hit distinct banks
  constexpr int KS = KC / 16;              // 16-wide k steps per chunk
  constexpr int ROWF4 = NT * 16 / EPU;     // 16-byte units per panel row
  constexpr int F4 = KC * ROWF4;
  constexpr int XPT = (F4 + NTHREADS - 1) / NTHREADS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  T* buf0 = lds;
  T* buf1 = lds + KC * LD;

  int first_tile, nseg = 1, c0, c1, slot = 0;
  bool partial = true;
  {
    const int b = blockIdx.x, C = sh.C;
    if (b < sh.whole) {
      first_tile = b; c0 = 0; c1 = C; partial = false;
    } else if (b < sh.whole + sh.lt * sh.f) {
      const int idx = b - sh.whole, s = idx % sh.f;
      first_tile = sh.whole + idx / sh.f;
      c0 = (int)((int64_t)s * (C - sh.x) / sh.f);
      c1 = (int)((int64_t)(s + 1) * (C - sh.x) / sh.f);
      slot = s;
    } else {
      const int i = b - sh.whole - sh.lt * sh.f;
      first_tile = sh.whole + i * sh.j;
      nseg = min(sh.j, sh.whole + sh.lt - first_tile);
      c0 = C - sh.x; c1 = C; slot = sh.f;
    }
  }
  const int nchunks = c1 - c0;
  const int kbeg = c0 * KC;
  const int kend = min(K, c1 * KC);
  const int K4 = K & ~3;
  const bool ragged = RAGGED && (K4 != K || K < 4);   // RAGGED = false: the launcher has checked K % 4 == 0, K >= 4

  for (int seg = 0; seg < nseg; ++seg) {
  const int row0 = (first_tile + seg) * (WAVES * MT * 16) + wave * (MT * 16);

  const T* ap[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int row = min(row0 + mt * 16 + r, rows - 1);
    ap[mt] = A + (int64_t)row * lda;
  }

  vec4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = vec4{T(0), T(0), T(0), T(0)};

  unit16 xr[XPT];
  vec4 a_cur[MT][KS], a_nxt[MT][KS];

#define LOAD_X(kbase)                                                              \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    int k = (kbase) + kr;                                                          \
    unit16 v = unit16{};                                                           \
    if (idx < F4 && k < kend) v = *(const unit16*)(X + (int64_t)k * ldx + c4 * EPU); \
    xr[i] = v;                                                                     \
  }
#define STORE_X(buf)                                                               \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    if (idx < F4) *(unit16*)((buf) + kr * LD + c4 * EPU) = xr[i];                  \
  }
  // A lane takes four consecutive k of its row with one load (rows may start at any element address).  Groups
  // past the end of a row whose length is a multiple of four are clamped to the last group: they meet zero
  // rows of the staged panel.  A row length that is not a multiple of four leaves a group that straddles the
  // end of the row; the chunk that holds it (one per row) is loaded element by element instead.
#define LOAD_A(dst, kbase)                                                         \
  if (ragged && (kbase) + KC > K4) {                                               \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                              \
    _Pragma("unroll") for (int s = 0; s < KS; ++s) {                               \
      const int k = (kbase) + s * 16 + 4 * g;                                      \
      _Pragma("unroll") for (int j = 0; j < 4; ++j)                                \
        dst[mt][s][j] = ap[mt][min(k + j, K - 1)];                                 \
    }                                                                              \
  } else {                                                                         \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                              \
    _Pragma("unroll") for (int s = 0; s < KS; ++s) {                               \
      const int k = min((kbase) + s * 16 + 4 * g, K - 4);                          \
      dst[mt][s] = *(const vec4u*)(ap[mt] + k);                                    \
    }                                                                              \
  }

  {
    LOAD_X(kbeg);
    LOAD_A(a_nxt, kbeg);
    STORE_X(buf0);
  }
  __syncthreads();

  // Not unrolled on purpose: the register copy a_cur = a_nxt at the top of an iteration is where the
  // wait for the prefetched block of A belongs; without it the compiler ends up waiting for the
  // freshly issued loads of the next chunk in the middle of the MFMA stream.
#pragma nounroll
  for (int c = 0; c < nchunks; ++c) {
    const T* cur = (c & 1) ? buf1 : buf0;
    T* nxt = (c & 1) ? buf0 : buf1;
    const bool more = (c + 1 < nchunks);
    // the block of A prefetched during the previous chunk becomes current (this copy is where
    // the wait for those loads sits), then the next one is requested
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int s = 0; s < KS; ++s) a_cur[mt][s] = opaque(a_nxt[mt][s]);
    if (more) {
      LOAD_X(kbeg + (c + 1) * KC);
      LOAD_A(a_nxt, kbeg + (c + 1) * KC);
    }
    // 4*KS steps of 4 contraction indices each; the panel values of step t+1 are read from LDS
    // while the MFMAs of step t run (register double buffer bq).
    {
      T bq[2][NT];
      const T* bbase = cur + (4 * g) * LD + r;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bq[0][nt] = bbase[nt * 16];
#pragma unroll
      for (int t = 0; t < 4 * KS; ++t) {
        if (t + 1 < 4 * KS) {
          const T* brow = bbase + (((t + 1) >> 2) * 16 + ((t + 1) & 3)) * LD;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) bq[(t + 1) & 1][nt] = brow[nt * 16];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads of step t+1 ahead of the MFMAs of step t
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt][nt] = mfma16(a_cur[mt][t >> 2][t & 3], bq[t & 1][nt], acc[mt][nt]);
      }
    }
    if (more) STORE_X(nxt);
    __syncthreads();
  }
#undef LOAD_X
#undef STORE_X
#undef LOAD_A

  // partial panels hold only the rows of the leftover tiles, i.e. rows from sh.whole tiles on
  const int part_row0 = sh.whole * (WAVES * MT * 16);
  T* Yo = partial ? Part + (int64_t)slot * split_stride - (int64_t)part_row0 * ldp : Y;
  const int64_t ldo = partial ? ldp : ldy;
  const int nc = partial ? NT * 16 : ncols;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      int row = row0 + mt * 16 + El<T>::acc_row(g, v);
      if (row < rows) {
        T* yr = Yo + (int64_t)row * ldo;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          int col = nt * 16 + r;
          if (col < nc) yr[col] = acc[mt][nt][v];
        }
      }
    }
  }   // next tail strip of this workgroup
}

// --------------------------------------------------------------------------------------------
// gemm_an for the narrowest panels (one column tile, l <= 16, fp32): bound by the read of A
// --------------------------------------------------------------------------------------------
// The MFMA A operand wants lane (r, g) to hold row r, so a load straight into the operand registers
// touches 16 rows with 64 bytes each per instruction, and a workgroup of k_gemm_an takes 256 bytes of a
// row per chunk.  Wide panels hide that behind the MFMAs; with a single column tile the kernel is a read
// of A, and how A is read decides: a plain read of a 76800 x 2000 matrix runs at 5.3 TB/s when every
// workgroup takes 256 bytes per row at a time and at 6.5 TB/s with 1 KiB per row.  Here a workgroup
// therefore owns 32 rows and walks them in chunks of 256 columns: a wave reads 1 KiB of one row per
// instruction (nontemporal), the block goes through LDS (row stride 260 words: the 16 lanes of a pass of
// a 128-bit LDS read hit 64 distinct banks), and the four waves split the chunk's columns, wave w
// multiplying columns [64 w, 64 w + 64) of all 32 rows; their four partial tiles are added in wave order
// at the end.  Both operands of a chunk are in registers before its MFMAs start, so block and panel
// chunk are single buffered in LDS and the stores of the next chunk overlap the MFMAs; two register sets
// hold the blocks of the next two chunks, i.e. a load has two chunk times to arrive.  Work partition
// (AnShape) and partial-panel convention are those of k_gemm_an with tiles of 32 rows and chunks of 256
// columns.  Measured (l = 16): 100000 x 50000 6.3 TB/s against 5.6 for k_gemm_an, 76800 x 2000 5.2 against
// 4.8.  With two column tiles the MFMA work doubles and this arrangement, whose MFMA phases do not overlap
// its LDS phases within a wave, loses to k_gemm_an (76800 x 2000, l = 20: 157 against 152 us), so it is
// instantiated for one tile only.
constexpr int kAnNarrowMaxNT = 1;
constexpr int kAnNarrowMinK = 512;   // shorter rows leave most of a 256-column chunk empty: k_gemm_an takes them
constexpr int kAnNarrowRows = 32;
constexpr int kAnNarrowKC = 256;
constexpr int kAnNarrowLDA = kAnNarrowKC + 4;
static constexpr int an_narrow_lds_bytes(int nt) {
  return (kAnNarrowRows * kAnNarrowLDA + kAnNarrowKC * (nt * 16 + 4)) * 4;
}

template <int NT, bool RAGGED>
__global__ void __launch_bounds__(256, 2)
k_gemm_an_narrow(const float* __restrict__ A, int64_t lda, int rows, int K,
                 const float* __restrict__ X, int ldx,
                 float* __restrict__ Y, int64_t ldy, int ncols,
                 float* __restrict__ Part, int64_t ldp, int64_t split_stride, AnShape sh) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);
  constexpr int MT = 2, KC = kAnNarrowKC, KS = 4, NTHREADS = 256, ROWS = kAnNarrowRows;
  constexpr int LD = NT * 16 + 4;
  constexpr int LDA = kAnNarrowLDA;
  constexpr int ROWF4 = NT * 4;              // 16-byte units per panel row
  constexpr int XPT = KC * ROWF4 / NTHREADS; // 4 or 8
  constexpr int APT = ROWS * (KC / 4) / NTHREADS;  // 16-byte units of A per thread and chunk (8)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  float* abuf = lds;
  float* xbuf = lds + ROWS * LDA;

  int first_tile, nseg = 1, c0, c1, slot = 0;
  bool partial = true;
  {
    const int b = blockIdx.x, C = sh.C;
    if (b < sh.whole) {
      first_tile = b; c0 = 0; c1 = C; partial = false;
    } else if (b < sh.whole + sh.lt * sh.f) {
      const int idx = b - sh.whole, sp = idx % sh.f;
      first_tile = sh.whole + idx / sh.f;
      c0 = (int)((int64_t)sp * (C - sh.x) / sh.f);
      c1 = (int)((int64_t)(sp + 1) * (C - sh.x) / sh.f);
      slot = sp;
    } else {
      const int i = b - sh.whole - sh.lt * sh.f;
      first_tile = sh.whole + i * sh.j;
      nseg = min(sh.j, sh.whole + sh.lt - first_tile);
      c0 = C - sh.x; c1 = C; slot = sh.f;
    }
  }
  const int nchunks = c1 - c0;
  const int kbeg = c0 * KC;
  const int kend = min(K, c1 * KC);
  const int K4 = K & ~3;
  const bool ragged = RAGGED && (K4 != K || K < 4);
  typedef floatx4 floatx4u __attribute__((aligned(4)));

  for (int seg = 0; seg < nseg; ++seg) {
  const int tile0 = (first_tile + seg) * ROWS;

  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

  floatx4 xr[XPT], ra[APT], rb[APT], a_cur[MT][KS];
  float b_cur[4 * KS][NT];

#define LOAD_X(kbase)                                                              \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    int k = (kbase) + kr;                                                          \
    floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};                                       \
    if (k < kend) v = *(const floatx4*)(X + (int64_t)k * ldx + c4 * 4);            \
    xr[i] = v;                                                                     \
  }
#define STORE_X()                                                                  \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    *(floatx4*)(xbuf + kr * LD + c4 * 4) = xr[i];                                  \
  }
  // a wave reads 1 KiB of one row per instruction (rows may start at any element address); columns past the
  // end of the row are re-read from its last ones: they meet zero rows of the staged panel.  The one chunk of
  // a row whose length is not a multiple of four that holds the straddling group is loaded element by element.
#define LOAD_A(dst, kbase)                                                         \
  _Pragma("unroll") for (int i = 0; i < APT; ++i) {                                \
    const int row = min(tile0 + wave + 4 * i, rows - 1);                           \
    const float* ap = A + (int64_t)row * lda;                                      \
    const int k = (kbase) + 4 * lane;                                              \
    if (ragged && (kbase) + KC > K4) {                                             \
      _Pragma("unroll") for (int j = 0; j < 4; ++j)                                \
        dst[i][j] = ap[min(k + j, K - 1)];                                         \
    } else {                                                                       \
      dst[i] = BRSVD_LOAD_A((const floatx4u*)(ap + min(k, K - 4)));             \
    }                                                                              \
  }
#define STORE_A(src)                                                               \
  _Pragma("unroll") for (int i = 0; i < APT; ++i)                                  \
    *(floatx4*)(abuf + (wave + 4 * i) * LDA + 4 * lane) = src[i];
  // operands of this wave's quarter of the chunk: columns [64 wave, 64 wave + 64)
#define READ_OPERANDS()                                                            \
  _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                \
  _Pragma("unroll") for (int s = 0; s < KS; ++s)                                   \
    a_cur[mt][s] = *(const floatx4*)(abuf + (mt * 16 + r) * LDA + 64 * wave + 16 * s + 4 * g); \
  _Pragma("unroll") for (int t = 0; t < 4 * KS; ++t)                               \
  _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                \
    b_cur[t][nt] = xbuf[(64 * wave + (t >> 2) * 16 + 4 * g + (t & 3)) * LD + nt * 16 + r];
  // One chunk: the panel rows of chunk c + 1 are requested (they come from L2 while the operands of chunk c
  // leave LDS), the staged copies of chunk c + 1 (block of A from the register set `rs`, panel rows from xr)
  // take the operands' place, the loads of chunk c + 3 are issued into the set just emptied, then the MFMAs
  // of chunk c run from registers.
#define CHUNK(c, rs)                                                               \
  {                                                                                \
    if ((c) + 1 < nchunks) LOAD_X(kbeg + ((c) + 1) * KC);                          \
    READ_OPERANDS();                                                               \
    __syncthreads();                                                               \
    if ((c) + 1 < nchunks) { STORE_A(rs); STORE_X(); }                             \
    if ((c) + 3 < nchunks) LOAD_A(rs, kbeg + ((c) + 3) * KC);                      \
    _Pragma("unroll") for (int t = 0; t < 4 * KS; ++t)                             \
    _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                              \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                              \
      acc[mt][nt] = mfma16(a_cur[mt][t >> 2][t & 3], b_cur[t][nt], acc[mt][nt]);   \
    __syncthreads();                                                               \
  }

  LOAD_X(kbeg);
  LOAD_A(ra, kbeg);
  if (nchunks > 1) LOAD_A(rb, kbeg + KC);
  STORE_X();
  STORE_A(ra);
  if (nchunks > 2) LOAD_A(ra, kbeg + 2 * KC);
  __syncthreads();
#pragma nounroll
  for (int c = 0; c < nchunks; c += 2) {
    CHUNK(c, rb);
    if (c + 1 < nchunks) CHUNK(c + 1, ra);
  }
#undef LOAD_X
#undef STORE_X
#undef LOAD_A
#undef STORE_A
#undef READ_OPERANDS
#undef CHUNK

  // the four partial tiles (one per wave, each over a quarter of every chunk) are added in wave order;
  // the staging area of the block is free after the last barrier of the chunk loop
  float* red = abuf;                                   // [wave][32 rows][NT * 16]
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        red[(wave * ROWS + mt * 16 + 4 * g + v) * (NT * 16) + nt * 16 + r] = acc[mt][nt][v];
  __syncthreads();
  {
    const int part_row0 = sh.whole * ROWS;
    float* Yo = partial ? Part + (int64_t)slot * split_stride - (int64_t)part_row0 * ldp : Y;
    const int64_t ldo = partial ? ldp : ldy;
    const int nc = partial ? NT * 16 : ncols;
    for (int e = tid; e < ROWS * NT * 16; e += NTHREADS) {
      const int lr = e / (NT * 16), col = e - lr * (NT * 16);
      const int row = tile0 + lr;
      float sum = red[e];
#pragma unroll
      for (int w = 1; w < 4; ++w) sum += red[w * ROWS * NT * 16 + e];
      if (row < rows && col < nc) Yo[(int64_t)row * ldo + col] = sum;
    }
  }
  __syncthreads();                                     // before the next strip reuses the staging area
  }   // next tail strip of this workgroup
}

// --------------------------------------------------------------------------------------------
// gemm_at
// --------------------------------------------------------------------------------------------
// Workgroup: WAVES waves, wave w owns MT*16 consecutive columns of A (= rows of Z) and all NT*16
// panel columns; blockIdx.x = column tile, blockIdx.y = (row block, sub-range) of the contraction.
// A lane loads MT consecutive columns of one row; component j of that load is the A operand of
// m-tile j, which therefore holds the interleaved columns {cw + MT*i + j : i = 0..15}.
template <typename T, int NT, int MT, int WAVES, int KC, bool RAGGED>
__global__ void __launch_bounds__(WAVES * 64)
k_gemm_at(const T* __restrict__ A, int64_t lda, int64_t rows_total, int n,
          const T* __restrict__ Q, int ldq,
          T* __restrict__ Zpart, int ldz, int64_t split_stride,
          int64_t block_rows, int sub, int rows_per_sub) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  T* lds = reinterpret_cast<T*>(lds_raw);
  typedef typename El<T>::v4 vec4;
  typedef typename El<T>::u16 unit16;
  constexpr int EPU = El<T>::kPerU16;
  constexpr int BM = El<T>::kBankMod;
  constexpr int NTHREADS = WAVES * 64;
  constexpr int LD = NT * 16 + ((16 - (NT * 16) % BM) + BM) % BM;   // row stride = 16 elements mod the bank period
  constexpr int KS = KC / 4;               // 4-row k steps per chunk
  constexpr int ROWF4 = NT * 16 / EPU;     // 16-byte units per panel row
  constexpr int F4 = KC * ROWF4;
  constexpr int XPT = (F4 + NTHREADS - 1) / NTHREADS;
  typedef T vecT __attribute__((ext_vector_type(MT)));
  typedef vecT vecTu __attribute__((aligned(sizeof(T))));   // MT consecutive columns at any element address

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int cw = blockIdx.x * (WAVES * MT * 16) + wave * (MT * 16);
  const int blk = blockIdx.y / sub, si = blockIdx.y - blk * sub;
  const int64_t bstart = (int64_t)blk * block_rows;
  const int64_t rbeg = bstart + (int64_t)si * rows_per_sub;
  int64_t rend = bstart + min((int64_t)(si + 1) * rows_per_sub, block_rows);
  rend = min(rend, rows_total);
  const int nchunks = rbeg < rend ? (int)((rend - rbeg + KC - 1) / KC) : 0;

  // A lane takes its MT consecutive columns with one load; groups past column n are clamped to the last group
  // (their rows of Z are not stored).  When n is not a multiple of MT one group straddles the end of the rows:
  // the workgroup that owns it (the last column tile) loads element by element instead.
  const int n_whole = n - n % MT;
  const bool by_element = RAGGED && (n_whole != n || n < MT) && (int)(blockIdx.x + 1) * (WAVES * MT * 16) > n_whole;
  int col[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) col[j] = min(cw + MT * r + j, n - 1);
  if (!by_element) col[0] = min(cw + MT * r, n - MT);

  vec4 acc[MT][NT];
#pragma unroll
  for (int j = 0; j < MT; ++j)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[j][nt] = vec4{T(0), T(0), T(0), T(0)};

  unit16 xr[XPT];
  vecT a_cur[KS], a_nxt[KS];

#define LOAD_Q(rbase)                                                              \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    int64_t row = (rbase) + kr;                                                    \
    unit16 v = unit16{};                                                           \
    if (idx < F4 && row < rend) v = *(const unit16*)(Q + row * ldq + c4 * EPU);    \
    xr[i] = v;                                                                     \
  }
#define STORE_Q(buf)                                                               \
  _Pragma("unroll") for (int i = 0; i < XPT; ++i) {                                \
    int idx = tid + i * NTHREADS;                                                  \
    int kr = idx / ROWF4, c4 = idx - kr * ROWF4;                                   \
    if (idx < F4) *(unit16*)((buf) + kr * LD + c4 * EPU) = xr[i];                  \
  }
#define LOAD_A(dst, rbase)                                                         \
  _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                 \
    int64_t row = min((rbase) + s * 4 + g, rows_total - 1);                        \
    const T* p = A + row * lda;                                                \
    if (by_element) {                                                              \
      _Pragma("unroll") for (int j = 0; j < MT; ++j)                               \
        dst[s][j] = p[col[j]];                                                     \
    } else {                                                                       \
      dst[s] = BRSVD_LOAD_A((const vecTu*)(p + col[0]));                        \
    }                                                                              \
  }

  T* buf0 = lds;
  T* buf1 = lds + KC * LD;

  if (nchunks > 0) {
    LOAD_Q(rbeg);
    LOAD_A(a_nxt, rbeg);
    STORE_Q(buf0);
  }
  __syncthreads();

  // Not unrolled on purpose: the register copy a_cur = a_nxt at the top of an iteration is where the
  // wait for the prefetched block of A belongs; without it the compiler ends up waiting for the
  // freshly issued loads of the next chunk in the middle of the MFMA stream.
#pragma nounroll
  for (int c = 0; c < nchunks; ++c) {
    const T* cur = (c & 1) ? buf1 : buf0;
    T* nxt = (c & 1) ? buf0 : buf1;
    const bool more = (c + 1 < nchunks);
#pragma unroll
    for (int s = 0; s < KS; ++s) a_cur[s] = opaque(a_nxt[s]);   // wait for the prefetched rows here
    if (more) {
      LOAD_Q(rbeg + (int64_t)(c + 1) * KC);
      LOAD_A(a_nxt, rbeg + (int64_t)(c + 1) * KC);
    }
    // KS steps of 4 rows each; the panel values of step s+1 are read from LDS while the MFMAs of
    // step s run (register double buffer bq).
    {
      T bq[2][NT];
      const T* bbase = cur + g * LD + r;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bq[0][nt] = bbase[nt * 16];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if (s + 1 < KS) {
          const T* brow = bbase + (s + 1) * 4 * LD;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) bq[(s + 1) & 1][nt] = brow[nt * 16];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads of step s+1 ahead of the MFMAs of step s
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int j = 0; j < MT; ++j) acc[j][nt] = mfma16(a_cur[s][j], bq[s & 1][nt], acc[j][nt]);
      }
    }
    if (more) STORE_Q(nxt);
    __syncthreads();
  }
#undef LOAD_Q
#undef STORE_Q
#undef LOAD_A

  T* Zo = Zpart + (int64_t)blockIdx.y * split_stride;
#pragma unroll
  for (int j = 0; j < MT; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      int zr = cw + MT * El<T>::acc_row(g, v) + j;
      if (zr < n) {
        T* zp = Zo + (int64_t)zr * ldz + r;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) zp[nt * 16] = acc[j][nt][v];
      }
    }
}

// out[row][col] = (accumulate ? out : 0) + sum_s part[s][row][col], summed in split order.
template <typename T>
__global__ void k_reduce_splits(const T* __restrict__ part, int nsplit, int64_t split_stride,
                                int64_t rows, int ncols, int64_t ldi, T* __restrict__ out,
                                int64_t ldo, int accumulate) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * ncols) return;
  int64_t row = idx / ncols;
  int col = (int)(idx - row * ncols);
  const T* p = part + row * ldi + col;
  T s = accumulate ? out[row * ldo + col] : T(0);
  for (int i = 0; i < nsplit; ++i) s += p[(int64_t)i * split_stride];
  out[row * ldo + col] = s;
}

// The same sum for partial panels that are contiguous (all ldi columns summed, ldo == ldi): 16 bytes per
// thread, splits unrolled so that several loads are in flight.
template <typename T>
__global__ void __launch_bounds__(256)
k_reduce_splits_flat(const T* __restrict__ part, int nsplit, int64_t split_stride, int64_t count16,
                     T* __restrict__ out, int accumulate) {
  typedef typename El<T>::u16 unit16;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= count16) return;
  constexpr int EPU = El<T>::kPerU16;
  const T* p = part + idx * EPU;
  unit16 s = accumulate ? *(const unit16*)(out + idx * EPU) : unit16{};
#pragma unroll 8
  for (int i = 0; i < nsplit; ++i) s += *(const unit16*)(p + (int64_t)i * split_stride);
  *(unit16*)(out + idx * EPU) = s;
}

// In-place first level of a long split sum: slot g*fan <- sum of the slots [g*fan, min((g+1)*fan, nsplit))
// in slot order (blockIdx.y = g).  Each thread only touches its own element of every slot.
template <typename T>
__global__ void k_reduce_groups_inplace(T* __restrict__ part, int nsplit, int fan, int64_t split_stride,
                                        int64_t count) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= count) return;                 // count <= split_stride elements of every slot take part
  const int s0 = blockIdx.y * fan, s1 = min(nsplit, s0 + fan);
  T* p = part + idx;
  T s = p[(int64_t)s0 * split_stride];
  for (int i = s0 + 1; i < s1; ++i) s += p[(int64_t)i * split_stride];
  p[(int64_t)s0 * split_stride] = s;
}

template <typename T>
__global__ void k_pad_panel(const T* __restrict__ src, int64_t rows, int l, T* __restrict__ dst, int Lp) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * Lp) return;
  int64_t row = idx / Lp;
  int col = (int)(idx - row * Lp);
  dst[idx] = col < l ? src[row * l + col] : T(0);
}

template <typename T>
__global__ void k_unpad_panel(const T* __restrict__ src, int64_t rows, int Lp, int l, T* __restrict__ dst,
                              int accumulate) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * l) return;
  int64_t row = idx / l;
  int col = (int)(idx - row * l);
  T v = src[row * Lp + col];
  dst[idx] = accumulate ? dst[idx] + v : v;
}

// dst[c][row] = src[row][c], c < l; 32x32 tiles through LDS.
template <typename T>
__global__ void k_transpose_panel(const T* __restrict__ src, int64_t rows, int Lp, int l, T* __restrict__ dst) {
  __shared__ T tile[32][33];
  int64_t r0 = (int64_t)blockIdx.x * 32;
  int c0 = blockIdx.y * 32;
  int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 256 threads: ty = 0..7
  for (int i = ty; i < 32; i += 8) {
    int64_t row = r0 + i;
    int col = c0 + tx;
    tile[i][tx] = (row < rows && col < Lp) ? src[row * Lp + col] : T(0);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    int col = c0 + i;
    int64_t row = r0 + tx;
    if (col < l && row < rows) dst[(int64_t)col * rows + row] = tile[tx][i];
  }
}

// --------------------------------------------------------------------------------------------
// Host-side launch logic
// --------------------------------------------------------------------------------------------
// Number of workgroup slots of the chip for a kernel whose workgroups use lds_bytes of LDS and run
// at most wg_per_cu_regs per CU because of registers (a static estimate: the plan must not depend
// on a device query, because the workspace is sized on the host before any GPU call).
static bool verbose() {
  static const bool v = [] { const char* e = getenv("BRSVD_VERBOSE"); return e && atoi(e) > 0; }();
  return v;
}
constexpr int kNumCUs = 256;
constexpr int kLdsPerCU = 160 * 1024;
static int wg_slots(int lds_bytes, int wg_per_cu_regs) {
  int by_lds = lds_bytes > 0 ? kLdsPerCU / lds_bytes : wg_per_cu_regs;
  int per_cu = by_lds < wg_per_cu_regs ? by_lds : wg_per_cu_regs;
  if (per_cu < 1) per_cu = 1;
  return kNumCUs * per_cu;
}

// Picks how many ways to split the contraction so that tiles*splits workgroups fill whole rounds
// of `slots`, without drowning the pass in partial-sum traffic.  out_over_in = bytes of one
// partial output panel (written and re-read) relative to the bytes of A the launch reads;
// units = indivisible pieces of the contraction range; traffic_weight in (0, 1] discounts that
// traffic when the launch is bound by MFMA rather than by HBM.
static int pick_splits(int64_t tiles, int slots, int64_t units, double out_over_in, double traffic_weight) {
  int best = 1;
  double best_score = -1.0;
  const int smax = (int)std::min<int64_t>(units, 4096);   // long split sums are reduced in two levels
  for (int sp = 1; sp <= smax; ++sp) {
    const int64_t per = ceil_div(units, sp);
    const int64_t eff_sp = ceil_div(units, per);          // splits actually produced
    if (eff_sp != sp) continue;
    const double w = (double)tiles * sp;
    const double rounds = std::ceil(w / slots);
    // time model in units of one contraction piece: rounds * (pieces per workgroup + fill), against
    // the ideal tiles*units/slots, plus the partial panels (one write and one read each)
    double score = ((double)tiles * units / slots) / (rounds * ((double)per + 0.5));
    score /= (1.0 + traffic_weight * 2.0 * out_over_in * (sp > 1 ? sp : 0));
    if (score > best_score * 1.002) { best_score = score; best = sp; }
  }
  return best;
}

struct NGroups {
  int groups, nt;   // column groups per launch sequence, n-tiles per group
};
// esz = element size: fp64 accumulators take twice the registers, so a launch keeps 8 n-tiles at most.
static int max_nt(int esz) { return esz == 8 ? 8 : kMaxNT; }
static NGroups column_groups(int Lp, int esz) {
  int nt_total = Lp / 16;
  int groups = (nt_total + max_nt(esz) - 1) / max_nt(esz);
  int nt = (nt_total + groups - 1) / groups;
  return {groups, nt};
}

// ---- gemm_an ----
struct AnCfg {
  int mt, waves, kc, tile_rows;
};
// Tile shapes picked from sweeps on MI355X (see the launch templates below, which must agree).
constexpr int64_t kAnWideK = 1024;
static AnCfg an_cfg(int nt, int esz, int64_t K) {
  auto cfg = [](int mt, int waves, int kc) { return AnCfg{mt, waves, kc, waves * mt * 16}; };
  if (esz == 8) return cfg(nt >= 5 ? 1 : 2, 4, 32);   // wide fp64 panels: one m-tile per wave keeps two waves per SIMD
  // one column tile: bound by the read of A (k_gemm_an_narrow: tiles of 32 rows, chunks of 256 columns)
  if (nt <= kAnNarrowMaxNT && K >= kAnNarrowMinK) return AnCfg{2, 4, kAnNarrowKC, kAnNarrowRows};
  // eight waves share one staged panel chunk (half the staging per MFMA); short contractions keep four-wave
  // workgroups, i.e. twice as many of them, and so do panels of two column tiles, which are close to the read
  // bound: more, smaller workgroups per CU overlap their load waits better (76800 x 2000, l = 20: 152 -> 135 us;
  // 100000 x 50000, l = 32: 4.5 -> 5.3 TB/s)
  if (nt <= 8) return cfg(2, (K >= kAnWideK && nt > 2) ? 8 : 4, 64);
  return cfg(nt > 14 ? 1 : 2, 8, 32);
}
// Discount of partial-panel traffic: 1 for HBM-bound widths, smaller once 2*Lp/8 flop/B is past the ridge.
static double traffic_weight(int nt) { return nt <= 2 ? 1.0 : (nt <= 4 ? 0.6 : 0.3); }
// Workgroups per CU assumed when a launch is cut to fill the chip.  The registers alone would allow more of
// the narrowest kernels (four-wave k_gemm_an with one or two column tiles: 112-128 registers, four workgroups per
// CU; eight-wave k_gemm_at with one or two column tiles: 104-124 registers, two), but plans made for those counts
// cut the contraction finer, and the extra partial panels and shorter workgroups cost more than the occupancy
// gains on the named shapes (76800 x 2000, l = 20: 135 -> 140 us and 109 -> 114 us), so the estimates stay at two
// and one.  The two-wave k_gemm_at (short rows) has 104 / 132 / 156 / 184 registers for one to four column tiles.
static int an_wg_per_cu_regs(int esz, int waves) { return esz == 8 ? 2 : (waves == 8 ? 1 : 2); }
static int at_wg_per_cu_regs(int nt, int waves) {
  if (waves == 8) return 1;
  return nt == 1 ? 8 : (nt <= 3 ? 6 : 4);
}
struct AnPlan {
  int row_tiles, tile_rows, nsplit, wgs;      // nsplit = partial panels per leftover tile (0: none)
  AnShape sh;
};
// See AnShape.  Short contractions (the R^-1 applies and lifts: fewer than 16 chunks) and launches
// with very many tiles keep one whole tile per workgroup.
static AnPlan an_plan(int64_t rows, int64_t K, int nt, int esz) {
  AnCfg c = an_cfg(nt, esz, K);
  AnPlan p;
  p.tile_rows = c.tile_rows;
  p.row_tiles = (int)ceil_div(rows, p.tile_rows);
  const int T = p.row_tiles, C = (int)ceil_div(K, c.kc);
  const bool narrow = esz == 4 && nt <= kAnNarrowMaxNT && K >= kAnNarrowMinK;
  const int lds_bytes = narrow ? an_narrow_lds_bytes(nt) : 2 * c.kc * (nt * 16 + 4) * esz;
  const int S = wg_slots(lds_bytes, an_wg_per_cu_regs(esz, c.waves));
  AnShape sh = {C, T, 0, 1, 0, 0};
  // a split or a strip is worth its partial panel from about 512 columns on: 8 chunks of 64, 2 of 256
  const int min_piece = c.kc >= 256 ? 2 : 8, min_strip = c.kc >= 256 ? 1 : 4;
  if (C >= 2 * min_piece && T < 8 * S) {
    sh.whole = T / S * S;
    sh.lt = T - sh.whole;
    if (sh.lt > 0) {
      sh.f = std::max(1, std::min(S / sh.lt, C / min_piece));
      const int spare = S - sh.f * sh.lt;
      if (spare > 0) {
        sh.j = (int)ceil_div(sh.lt, spare);
        sh.x = C / (1 + sh.f * sh.j);          // j strips weigh one main split: (C - x) / f = j * x
        if (sh.x < min_strip) { sh.x = 0; sh.j = 0; }
      }
      if (sh.f == 1 && sh.x == 0) { sh.whole = T; sh.lt = 0; }
    }
  }
  p.sh = sh;
  p.nsplit = sh.lt > 0 ? sh.f + (sh.x > 0 ? 1 : 0) : 0;
  p.wgs = sh.whole + sh.lt * sh.f + (sh.x > 0 ? (int)ceil_div(sh.lt, sh.j) : 0);
  return p;
}

// Rows that take part in a split sum: those of the leftover tiles.
static int64_t an_partial_rows(const AnPlan& p, int64_t rows) {
  return p.nsplit > 0 ? rows - (int64_t)p.sh.whole * p.tile_rows : 0;
}

uint64_t gemm_an_scratch_bytes(int64_t rows, int64_t K, int Lp, int esz) {
  NGroups ng = column_groups(Lp, esz);
  AnPlan p = an_plan(rows, K, ng.nt, esz);
  return (uint64_t)p.nsplit * an_partial_rows(p, rows) * Lp * esz;
}

// The launch plans as plain numbers, for host-side checks of their invariants.
void gemm_an_plan_describe(int64_t rows, int64_t K, int Lp, int esz, int32_t out[12]) {
  NGroups ng = column_groups(Lp, esz);
  AnPlan p = an_plan(rows, K, ng.nt, esz);
  const int32_t v[12] = {p.tile_rows, p.row_tiles, p.sh.C, p.sh.whole, p.sh.lt, p.sh.f, p.sh.x, p.sh.j, p.nsplit, p.wgs,
                         ng.groups, ng.nt};
  for (int i = 0; i < 12; ++i) out[i] = v[i];
}

template <typename T, int NT, int MT, int WAVES, int KC, bool RAGGED>
static int launch_an_inst_r(const T* A, int64_t lda, int rows, int K, const T* X, int ldx, T* Y, int64_t ldy,
                          int ncols, T* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                          hipStream_t stream) {
  auto kern = k_gemm_an<T, NT, MT, WAVES, KC, RAGGED>;
  constexpr int lds_bytes = 2 * KC * (NT * 16 + 4) * (int)sizeof(T);
  static bool attr_set = false;
  if (!attr_set) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      lds_bytes));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(p.wgs), dim3(WAVES * 64), lds_bytes, stream, A, lda, rows, K, X, ldx, Y, ldy,
                     ncols, part, ldp, split_stride, p.sh);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

// Rows that start on 16-byte boundaries and hold a whole number of a lane's element groups take the kernels
// compiled without the element-by-element path for the group that straddles a row's end (and, where A is
// streamed, with nontemporal loads); any other layout takes the RAGGED instance.
template <typename T>
static bool rows_aligned(const T* A, int64_t lda, int64_t len, int group) {
  constexpr int per16 = 16 / (int)sizeof(T);
  return len % group == 0 && len >= group && lda % per16 == 0 && ((uintptr_t)A) % 16 == 0;
}

template <typename T, int NT, int MT, int WAVES, int KC>
static int launch_an_inst(const T* A, int64_t lda, int rows, int K, const T* X, int ldx, T* Y, int64_t ldy,
                          int ncols, T* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                          hipStream_t stream) {
  if (rows_aligned(A, lda, K, 4))
    return launch_an_inst_r<T, NT, MT, WAVES, KC, false>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride,
                                                         p, stream);
  return launch_an_inst_r<T, NT, MT, WAVES, KC, true>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p,
                                                      stream);
}

template <int NT, bool RAGGED>
static int launch_an_narrow_r(const float* A, int64_t lda, int rows, int K, const float* X, int ldx, float* Y,
                            int64_t ldy, int ncols, float* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                            hipStream_t stream) {
  auto kern = k_gemm_an_narrow<NT, RAGGED>;
  constexpr int lds_bytes = an_narrow_lds_bytes(NT);
  static bool attr_set = false;
  if (!attr_set) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(p.wgs), dim3(256), lds_bytes, stream, A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp,
                     split_stride, p.sh);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <int NT>
static int launch_an_narrow(const float* A, int64_t lda, int rows, int K, const float* X, int ldx, float* Y,
                            int64_t ldy, int ncols, float* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                            hipStream_t stream) {
  if (rows_aligned(A, lda, K, 4))
    return launch_an_narrow_r<NT, false>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p, stream);
  return launch_an_narrow_r<NT, true>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p, stream);
}

template <typename T, int NT>
static int launch_an_nt(const T* A, int64_t lda, int rows, int K, const T* X, int ldx, T* Y,
                        int64_t ldy, int ncols, T* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                        hipStream_t stream) {
  if constexpr (sizeof(T) == 8 && NT > 8) {
    return BRSVD_ERR_ARG;                     // never planned: column_groups keeps fp64 launches at 8 n-tiles
  } else {
    if constexpr (sizeof(T) == 4 && NT <= kAnNarrowMaxNT) {
      if (K >= kAnNarrowMinK)
        return launch_an_narrow<NT>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p, stream);
    }
    constexpr int MT = ((sizeof(T) == 8 && NT >= 5) || NT > 14) ? 1 : 2;
    constexpr int KC = (sizeof(T) == 8 || NT > 8) ? 32 : 64;
    if constexpr (sizeof(T) == 4 && NT <= 8) {
      if (K >= kAnWideK && NT > 2)
        return launch_an_inst<T, NT, MT, 8, KC>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p,
                                                stream);
    }
    constexpr int W = NT > 8 ? 8 : 4;
    return launch_an_inst<T, NT, MT, W, KC>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p, stream);
  }
}

#define BRSVD_NT_SWITCH(nt, CALL)                                                      \
  switch (nt) {                                                                        \
    case 1: return CALL(1); case 2: return CALL(2); case 3: return CALL(3);            \
    case 4: return CALL(4); case 5: return CALL(5); case 6: return CALL(6);            \
    case 7: return CALL(7); case 8: return CALL(8); case 9: return CALL(9);            \
    case 10: return CALL(10); case 11: return CALL(11); case 12: return CALL(12);      \
    case 13: return CALL(13); case 14: return CALL(14); case 15: return CALL(15);      \
    case 16: return CALL(16); case 17: return CALL(17);                                \
    default: return BRSVD_ERR_ARG;                                                     \
  }

template <typename T>
static int launch_an(int nt, const T* A, int64_t lda, int rows, int K, const T* X, int ldx, T* Y,
                     int64_t ldy, int ncols, T* part, int64_t ldp, int64_t split_stride, const AnPlan& p,
                     hipStream_t stream) {
#define CALL(N) launch_an_nt<T, N>(A, lda, rows, K, X, ldx, Y, ldy, ncols, part, ldp, split_stride, p, stream)
  BRSVD_NT_SWITCH(nt, CALL)
#undef CALL
}

// Sum of the split partial panels in split order; long sums (more than kReduceFan splits) are taken in
// two levels, groups of kReduceFan consecutive splits first, so that no thread walks thousands of
// slots serially.  Either way the association is fixed by the plan, not by timing.
constexpr int kReduceFan = 16;
template <typename T>
static int reduce_splits(T* part, int nsplit, int64_t split_stride, int64_t rows, int ncols, int64_t ldi, T* out,
                         int64_t ldo, bool accumulate, hipStream_t stream) {
  int64_t total = rows * ncols;
  if (total == 0) return BRSVD_OK;
  if (nsplit > 2 * kReduceFan) {
    const int groups = (int)ceil_div(nsplit, kReduceFan);
    const int64_t count = rows * ldi;       // the rows being reduced, all ldi columns of each
    hipLaunchKernelGGL(k_reduce_groups_inplace<T>, dim3((unsigned)ceil_div(count, 256), groups), dim3(256), 0, stream,
                       part, nsplit, kReduceFan, split_stride, count);
    nsplit = groups;
    split_stride *= kReduceFan;
  }
  constexpr int EPU = 16 / (int)sizeof(T);
  const bool flat = ncols == ldi && ldo == ldi && total % EPU == 0 && split_stride % EPU == 0 &&
                    ((uintptr_t)part) % 16 == 0 && ((uintptr_t)out) % 16 == 0;
  if (flat)
    hipLaunchKernelGGL(k_reduce_splits_flat<T>, dim3((unsigned)ceil_div(total / EPU, 256)), dim3(256), 0, stream, part,
                       nsplit, split_stride, total / EPU, out, accumulate ? 1 : 0);
  else
    hipLaunchKernelGGL(k_reduce_splits<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                       part, nsplit, split_stride, rows, ncols, ldi, out, ldo, accumulate ? 1 : 0);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T>
static int gemm_an_t(const T* A, int64_t lda, int64_t rows, int64_t K, const T* X, int Lp, T* Y, int64_t ldy,
                     int ncols, void* scratch, uint64_t scratch_bytes, hipStream_t stream, const KernelEvents* ev) {
  if (rows <= 0 || K <= 0 || Lp <= 0 || Lp % 16 || ncols <= 0 || ncols > Lp) return BRSVD_ERR_ARG;
  if (rows > INT32_MAX || K > INT32_MAX) return BRSVD_ERR_ARG;
  constexpr int esz = (int)sizeof(T);
  NGroups ng = column_groups(Lp, esz);
  AnPlan p = an_plan(rows, K, ng.nt, esz);
  const int64_t prows = an_partial_rows(p, rows);
  if (scratch_bytes < (uint64_t)p.nsplit * prows * Lp * esz) return BRSVD_ERR_BUDGET;
  if (verbose())
    fprintf(stderr, "[brsvd] gemm_an f%d rows=%ld K=%ld Lp=%d: %d whole tiles + %d leftover tiles x %d splits + tail of %d "
            "chunks (%d per workgroup), %d chunks per tile, %d workgroups\n", esz * 8, (long)rows, (long)K, Lp,
            p.sh.whole, p.sh.lt, p.sh.f, p.sh.x, p.sh.j, p.sh.C, p.wgs);
  T* part = (T*)scratch;
  if (ev) BRSVD_HIP_TRY(hipEventRecord(ev->start, stream));
  for (int gi = 0; gi < ng.groups; ++gi) {
    int c0 = gi * ng.nt * 16;
    int nt = (Lp - c0) / 16 < ng.nt ? (Lp - c0) / 16 : ng.nt;
    if (nt <= 0) break;
    int nc = ncols - c0 < nt * 16 ? ncols - c0 : nt * 16;   // valid output columns in this group (may be <= 0)
    BRSVD_TRY(launch_an<T>(nt, A, lda, (int)rows, (int)K, X + c0, Lp, Y + c0, ldy, nc, part ? part + c0 : nullptr,
                           Lp, prows * Lp, p, stream));
  }
  if (ev) {
    BRSVD_HIP_TRY(hipEventRecord(ev->stop, stream));
    BRSVD_HIP_TRY(hipEventRecord(ev->sum_start, stream));
  }
  if (p.nsplit > 0) {
    // rows of the leftover tiles: their partial panels, in split order
    const int64_t r0 = rows - prows;
    BRSVD_TRY(reduce_splits<T>(part, p.nsplit, prows * Lp, prows, ncols, Lp, Y + r0 * ldy, ldy, false, stream));
  }
  if (ev) BRSVD_HIP_TRY(hipEventRecord(ev->sum_stop, stream));
  return BRSVD_OK;
}
int gemm_an(const float* A, int64_t lda, int64_t rows, int64_t K, const float* X, int Lp, float* Y, int64_t ldy,
            int ncols, void* scratch, uint64_t scratch_bytes, hipStream_t stream, const KernelEvents* ev) {
  return gemm_an_t<float>(A, lda, rows, K, X, Lp, Y, ldy, ncols, scratch, scratch_bytes, stream, ev);
}
int gemm_an(const double* A, int64_t lda, int64_t rows, int64_t K, const double* X, int Lp, double* Y, int64_t ldy,
            int ncols, void* scratch, uint64_t scratch_bytes, hipStream_t stream, const KernelEvents* ev) {
  return gemm_an_t<double>(A, lda, rows, K, X, Lp, Y, ldy, ncols, scratch, scratch_bytes, stream, ev);
}

// ---- gemm_at ----
struct AtPlan {
  int mt, waves, col_tiles, nblocks, sub, rows_per_sub, nsplit;
};
static int at_mt(int nt, int esz) { return (esz == 4 && nt <= 8) ? 4 : 2; }
constexpr int kAtWaves = 8;
constexpr int kAtKC = 32;
// Narrow A (tall-skinny inputs, n of a few hundred at most) with a narrow panel: workgroups of two
// waves (128 columns), so that no wave multiplies clamped duplicate columns and the row range can be
// cut into enough workgroups to fill the chip.
constexpr int kAtNarrowWaves = 2;
constexpr int kAtNarrowMaxNT = 4;
constexpr int kAtNarrowMaxN = 256;
static int at_waves(int64_t n, int nt, int esz) {
  return (esz == 4 && nt <= kAtNarrowMaxNT && n <= kAtNarrowMaxN) ? kAtNarrowWaves : kAtWaves;
}
static int at_ld(int nt, int esz) {
  const int bm = esz == 8 ? 32 : 64;
  return nt * 16 + ((16 - (nt * 16) % bm) + bm) % bm;
}

static AtPlan at_plan(int64_t rows, int64_t n, int nt, int64_t block_rows, int esz) {
  AtPlan p;
  p.mt = at_mt(nt, esz);
  p.waves = at_waves(n, nt, esz);
  p.col_tiles = (int)ceil_div(n, p.waves * p.mt * 16);
  if (block_rows <= 0 || block_rows > rows) block_rows = rows;
  p.nblocks = (int)ceil_div(rows, block_rows);
  const int max_sub = (int)ceil_div(block_rows, kAtKC);
  const int lds_bytes = 2 * kAtKC * at_ld(nt, esz) * esz;
  // one partial panel (n x Lp) per split, against block_rows x n of A read per block
  const int want = pick_splits((int64_t)p.col_tiles * p.nblocks, wg_slots(lds_bytes, at_wg_per_cu_regs(nt, p.waves)), max_sub,
                               (double)(nt * 16) / (double)block_rows, traffic_weight(nt));
  int64_t rps = ceil_div(block_rows, want);
  rps = ceil_div(rps, kAtKC) * kAtKC;
  p.rows_per_sub = (int)rps;
  p.sub = (int)ceil_div(block_rows, rps);
  p.nsplit = p.nblocks * p.sub;
  return p;
}

uint64_t gemm_at_scratch_bytes(int64_t rows, int64_t n, int Lp, int64_t block_rows, int esz) {
  NGroups ng = column_groups(Lp, esz);
  AtPlan p = at_plan(rows, n, ng.nt, block_rows, esz);
  return (uint64_t)p.nsplit * n * Lp * esz;
}

void gemm_at_plan_describe(int64_t rows, int64_t n, int Lp, int64_t block_rows, int esz, int32_t out[12]) {
  if (block_rows <= 0 || block_rows > rows) block_rows = rows;
  NGroups ng = column_groups(Lp, esz);
  AtPlan p = at_plan(rows, n, ng.nt, block_rows, esz);
  const int32_t v[12] = {p.mt, p.waves, p.col_tiles, p.nblocks, p.sub, p.rows_per_sub, p.nsplit, kAtKC, ng.groups, ng.nt, 0, 0};
  for (int i = 0; i < 12; ++i) out[i] = v[i];
}

template <typename T, int NT, int MT, int WAVES, bool RAGGED>
static int launch_at_inst_r(const T* A, int64_t lda, int64_t rows, int n, const T* Q, int ldq, T* Zp, int ldz,
                          int64_t split_stride, int64_t block_rows, const AtPlan& p, hipStream_t stream) {
  auto kern = k_gemm_at<T, NT, MT, WAVES, kAtKC, RAGGED>;
  constexpr int BM = El<T>::kBankMod;
  constexpr int LD = NT * 16 + ((16 - (NT * 16) % BM) + BM) % BM;
  constexpr int lds_bytes = 2 * kAtKC * LD * (int)sizeof(T);
  static bool attr_set = false;
  if (!attr_set) {
    BRSVD_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      lds_bytes));
    attr_set = true;
  }
  dim3 grid(p.col_tiles, p.nsplit);
  hipLaunchKernelGGL(kern, grid, dim3(WAVES * 64), lds_bytes, stream, A, lda, rows, n, Q, ldq, Zp, ldz,
                     split_stride, block_rows, p.sub, p.rows_per_sub);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template <typename T, int NT, int MT, int WAVES>
static int launch_at_inst(const T* A, int64_t lda, int64_t rows, int n, const T* Q, int ldq, T* Zp, int ldz,
                          int64_t split_stride, int64_t block_rows, const AtPlan& p, hipStream_t stream) {
  // short rows whose pitch is not a whole number of 128-byte lines share a line with the next row at both ends:
  // they are read with the plain loads of the RAGGED instance (2073600 x 100: 281 -> 265 us per pass)
  const int64_t pitch = lda * (int64_t)sizeof(T);
  if (rows_aligned(A, lda, n, MT) && (pitch % 128 == 0 || pitch >= 2048))
    return launch_at_inst_r<T, NT, MT, WAVES, false>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p, stream);
  return launch_at_inst_r<T, NT, MT, WAVES, true>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p, stream);
}

template <typename T, int NT>
static int launch_at_nt(const T* A, int64_t lda, int64_t rows, int n, const T* Q, int ldq, T* Zp,
                        int ldz, int64_t split_stride, int64_t block_rows, const AtPlan& p, hipStream_t stream) {
  if constexpr (sizeof(T) == 8) {
    if constexpr (NT > 8) {
      return BRSVD_ERR_ARG;
    } else {
      return launch_at_inst<T, NT, 2, kAtWaves>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p, stream);
    }
  } else {
    constexpr int MT = NT <= 8 ? 4 : 2;
    if constexpr (NT <= kAtNarrowMaxNT) {
      if (p.waves == kAtNarrowWaves)
        return launch_at_inst<T, NT, MT, kAtNarrowWaves>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p,
                                                         stream);
    }
    return launch_at_inst<T, NT, MT, kAtWaves>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p, stream);
  }
}

template <typename T>
static int launch_at(int nt, const T* A, int64_t lda, int64_t rows, int n, const T* Q, int ldq, T* Zp,
                     int ldz, int64_t split_stride, int64_t block_rows, const AtPlan& p, hipStream_t stream) {
#define CALL(N) launch_at_nt<T, N>(A, lda, rows, n, Q, ldq, Zp, ldz, split_stride, block_rows, p, stream)
  BRSVD_NT_SWITCH(nt, CALL)
#undef CALL
}

template <typename T>
static int gemm_at_t(const T* A, int64_t lda, int64_t rows, int64_t n, const T* Q, int Lp, T* Z, bool accumulate,
                     int64_t block_rows, void* scratch, uint64_t scratch_bytes, hipStream_t stream,
                     const KernelEvents* ev) {
  if (rows <= 0 || n <= 0 || Lp <= 0 || Lp % 16) return BRSVD_ERR_ARG;
  if (n > INT32_MAX) return BRSVD_ERR_ARG;
  if (block_rows <= 0 || block_rows > rows) block_rows = rows;
  constexpr int esz = (int)sizeof(T);
  NGroups ng = column_groups(Lp, esz);
  AtPlan p = at_plan(rows, n, ng.nt, block_rows, esz);
  if (p.nsplit > 65535) return BRSVD_ERR_ARG;
  if (scratch_bytes < (uint64_t)p.nsplit * n * Lp * esz) return BRSVD_ERR_BUDGET;
  T* part = (T*)scratch;
  if (verbose())
    fprintf(stderr, "[brsvd] gemm_at f%d rows=%ld n=%ld Lp=%d: %d col tiles (%d waves) x %d blocks x %d sub-ranges of %d rows\n",
            esz * 8, (long)rows, (long)n, Lp, p.col_tiles, p.waves, p.nblocks, p.sub, p.rows_per_sub);
  if (ev) BRSVD_HIP_TRY(hipEventRecord(ev->start, stream));
  for (int gi = 0; gi < ng.groups; ++gi) {
    int c0 = gi * ng.nt * 16;
    int nt = (Lp - c0) / 16 < ng.nt ? (Lp - c0) / 16 : ng.nt;
    if (nt <= 0) break;
    BRSVD_TRY(launch_at<T>(nt, A, lda, rows, (int)n, Q + c0, Lp, part + c0, Lp, n * Lp, block_rows, p, stream));
  }
  if (ev) {
    BRSVD_HIP_TRY(hipEventRecord(ev->stop, stream));
    BRSVD_HIP_TRY(hipEventRecord(ev->sum_start, stream));
  }
  BRSVD_TRY(reduce_splits<T>(part, p.nsplit, n * Lp, n, Lp, Lp, Z, Lp, accumulate, stream));
  if (ev) BRSVD_HIP_TRY(hipEventRecord(ev->sum_stop, stream));
  return BRSVD_OK;
}
int gemm_at(const float* A, int64_t lda, int64_t rows, int64_t n, const float* Q, int Lp, float* Z, bool accumulate,
            int64_t block_rows, void* scratch, uint64_t scratch_bytes, hipStream_t stream, const KernelEvents* ev) {
  return gemm_at_t<float>(A, lda, rows, n, Q, Lp, Z, accumulate, block_rows, scratch, scratch_bytes, stream, ev);
}
int gemm_at(const double* A, int64_t lda, int64_t rows, int64_t n, const double* Q, int Lp, double* Z, bool accumulate,
            int64_t block_rows, void* scratch, uint64_t scratch_bytes, hipStream_t stream, const KernelEvents* ev) {
  return gemm_at_t<double>(A, lda, rows, n, Q, Lp, Z, accumulate, block_rows, scratch, scratch_bytes, stream, ev);
}

template <typename T>
static int pad_panel_t(const T* src, int64_t rows, int l, T* dst, int Lp, hipStream_t stream) {
  int64_t total = rows * Lp;
  hipLaunchKernelGGL(k_pad_panel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, src, rows, l, dst, Lp);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}
template <typename T>
static int unpad_panel_t(const T* src, int64_t rows, int Lp, int l, T* dst, bool accumulate, hipStream_t stream) {
  int64_t total = rows * l;
  hipLaunchKernelGGL(k_unpad_panel<T>, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream, src, rows, Lp, l,
                     dst, accumulate ? 1 : 0);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}
template <typename T>
static int transpose_panel_t(const T* src, int64_t rows, int Lp, int l, T* dst, hipStream_t stream) {
  dim3 grid((unsigned)ceil_div(rows, 32), (unsigned)ceil_div(l, 32));
  hipLaunchKernelGGL(k_transpose_panel<T>, grid, dim3(256), 0, stream, src, rows, Lp, l, dst);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}
int pad_panel(const float* s, int64_t rows, int l, float* d, int Lp, hipStream_t st) { return pad_panel_t(s, rows, l, d, Lp, st); }
int pad_panel(const double* s, int64_t rows, int l, double* d, int Lp, hipStream_t st) { return pad_panel_t(s, rows, l, d, Lp, st); }
int unpad_panel(const float* s, int64_t rows, int Lp, int l, float* d, bool acc, hipStream_t st) {
  return unpad_panel_t(s, rows, Lp, l, d, acc, st);
}
int unpad_panel(const double* s, int64_t rows, int Lp, int l, double* d, bool acc, hipStream_t st) {
  return unpad_panel_t(s, rows, Lp, l, d, acc, st);
}
int transpose_panel(const float* s, int64_t rows, int Lp, int l, float* d, hipStream_t st) {
  return transpose_panel_t(s, rows, Lp, l, d, st);
}
int transpose_panel(const double* s, int64_t rows, int Lp, int l, double* d, hipStream_t st) {
  return transpose_panel_t(s, rows, Lp, l, d, st);
}

}  // namespace brsvd
