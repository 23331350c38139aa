// Driver and C ABI of libbrsvd: the block randomized SVD of Alg. 1 / Alg. 2 on one MI355X.
//
// Pass structure (l = k + p, A visited in row blocks; "pass" = one full read of A):
//   pass 0          Y = A * Omega                 gemm_an     Q = orth(Y)
//   q times         Z = A^T * Q                   gemm_at     W = orth(Z)
//                   Y = A * W                     gemm_an     Q = orth(Y)
//   last pass       B^T = A^T * Q                 gemm_at     B^T = W_B * R_B (orth, R kept)
//   small SVD       R_B = Ur diag(s) Vr^T         Jacobi
//   lifts           U = Q * Vr,  V = W_B * Ur, V^T stored
// Device-resident A: each pass is one launch over all rows (the row blocks matter only when A is
// streamed, and in the block-local scheme).  Host-resident A: each block is copied into one of two
// staging buffers on the copy stream while the other is being multiplied on the compute stream.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "brsvd_steps.h"
#include "common.h"

using namespace brsvd;

namespace {

constexpr uint64_t kAlign = 256;
constexpr uint64_t align_up(uint64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

enum Cat { CAT_AN = 0, CAT_AT, CAT_ORTH, CAT_SVD, CAT_LIFT, CAT_COPY, CAT_ELEM, CAT_TOTAL, CAT_SUM, CAT_UPD, CAT_COUNT };

struct Layout {
  // offsets into the arena
  uint64_t Pm[2], Pn[2], gemm_scratch, gram_part, G, R0, R1, Xinv, Rinv, Rtot, XV, XU, svdW, svdJ, sig,
      S32, flags, tsqr, stage[2], scal, rpcaU, rpcaVt, rpca_part, total;
  uint64_t gemm_scratch_bytes, tsqr_bytes, stage_bytes;
  int gram_chunks;
};

}  // namespace

struct brsvd_handle_s {
  brsvd_params prm;
  int l, Lp;
  int64_t b;
  int nblocks;
  bool host_a;
  Layout lay;
  char* arena;
  hipStream_t compute, copy;
  bool own_copy;
  hipEvent_t filled[2], drained[2];
  int* host_flags;                 // pinned: [0] breakdown, [1] sweeps, [2] converged
  double* host_scal;               // pinned scalars for the robust-PCA loop
  std::vector<hipEvent_t> ev;      // timing event pool
  std::vector<std::pair<int, int>> regions[CAT_COUNT];
  size_t ev_used;
  bool timing;
  bool own_arena;                  // false: the arena is the caller's workspace
  int64_t launches[CAT_COUNT];
  int64_t bytes_A_kernels;         // bytes of A (or of its staged blocks) read by the pass kernels
  int64_t bytes_A_copied;          // bytes of A copied host -> device

  int esz() const { return prm.dtype == BRSVD_DTYPE_F64 ? 8 : 4; }
  template <typename T = float> T* Pm(int i) { return (T*)(arena + lay.Pm[i]); }
  template <typename T = float> T* Pn(int i) { return (T*)(arena + lay.Pn[i]); }
  template <typename T> T* at(uint64_t off) { return (T*)(arena + off); }
};

namespace {

int validate(const brsvd_params* p) {
  if (!p) return BRSVD_ERR_ARG;
  if (p->m < 1 || p->n < 1 || p->k < 1 || p->p < 0 || p->q < 0) return BRSVD_ERR_ARG;
  int64_t l = (int64_t)p->k + p->p;
  if (l > kMaxL || l > p->m || l > p->n) return BRSVD_ERR_ARG;
  if (p->m > INT32_MAX || p->n > INT32_MAX) return BRSVD_ERR_ARG;
  if (p->a_location != BRSVD_A_DEVICE && p->a_location != BRSVD_A_HOST_PINNED) return BRSVD_ERR_ARG;
  if (p->orth_method < BRSVD_ORTH_AUTO || p->orth_method > BRSVD_ORTH_TSQR) return BRSVD_ERR_ARG;
  if (p->row_block < 0) return BRSVD_ERR_ARG;
  if (p->pass_mode != BRSVD_PASSES_SEPARATE && p->pass_mode != BRSVD_PASSES_FUSED) return BRSVD_ERR_ARG;
  if (p->dtype != BRSVD_DTYPE_F32 && p->dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  if (p->timing_level != 0 && p->timing_level != 1) return BRSVD_ERR_ARG;
  if (p->workspace && ((uintptr_t)p->workspace) % kAlign != 0) return BRSVD_ERR_ARG;
  return BRSVD_OK;
}

// Working set for a given row block b.
Layout make_layout(const brsvd_params& p, int64_t b) {
  Layout L;
  std::memset(&L, 0, sizeof(L));
  const int l = p.k + p.p, Lp = padded_l(l);
  const int64_t m = p.m, n = p.n;
  const bool host = p.a_location == BRSVD_A_HOST_PINNED;
  const int esz = p.dtype == BRSVD_DTYPE_F64 ? 8 : 4;      // element size of A and of the panels
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += align_up(bytes); return o; };
  for (int i = 0; i < 2; ++i) L.Pm[i] = take((uint64_t)m * Lp * esz);
  for (int i = 0; i < 2; ++i) L.Pn[i] = take((uint64_t)n * Lp * esz);
  // split-sum scratch: the largest of every GEMM shape issued by the driver
  uint64_t gs = 0;
  // products on one row block (streamed A, and the block-local scheme on any A), also on a ragged last block
  for (int64_t rows : {b, m - (m - 1) / b * b}) {
    gs = std::max(gs, gemm_an_scratch_bytes(rows, n, Lp, esz));
    gs = std::max(gs, gemm_at_scratch_bytes(rows, n, Lp, rows, esz));
  }
  if (!host) {   // device-resident A: one launch over all rows
    gs = std::max(gs, gemm_an_scratch_bytes(m, n, Lp, esz));
    gs = std::max(gs, gemm_at_scratch_bytes(m, n, Lp, m, esz));
  }
  if (!host) {   // single-vector products of the spectral-norm power method (16-column panels)
    gs = std::max(gs, gemm_an_scratch_bytes(m, n, kTile, esz));
    gs = std::max(gs, gemm_at_scratch_bytes(m, n, kTile, m, esz));
  }
  gs = std::max(gs, gemm_an_scratch_bytes(m, Lp, Lp, esz));
  gs = std::max(gs, gemm_an_scratch_bytes(n, Lp, Lp, esz));
  L.gemm_scratch_bytes = gs;
  L.gemm_scratch = take(gs);
  L.gram_chunks = (int)std::max(orth_gram_slots(m, Lp), orth_gram_slots(n, Lp));
  L.gram_part = take((uint64_t)L.gram_chunks * Lp * Lp * 8);
  const uint64_t sq8 = (uint64_t)Lp * Lp * 8;
  L.G = take(sq8); L.R0 = take(sq8); L.R1 = take(sq8); L.Xinv = take(sq8); L.Rtot = take(sq8);
  const uint64_t sqe = (uint64_t)Lp * Lp * esz;
  L.Rinv = take(sqe); L.XV = take(sqe); L.XU = take(sqe);
  L.svdW = take(sq8); L.svdJ = take(sq8);
  L.sig = take((uint64_t)3 * Lp * 8);
  L.S32 = take((uint64_t)Lp * esz);
  L.flags = take(64);
  L.scal = take(64);
  if (!host) {   // results of the inner SVDs of the robust-PCA loop, and its reduction scratch
    L.rpcaU = take((uint64_t)m * l * esz);
    L.rpcaVt = take((uint64_t)l * n * esz);
    L.rpca_part = take(rpca_part_doubles(m, n) * 8);
  }
  L.tsqr_bytes = std::max(tsqr_work_bytes(m, Lp), tsqr_work_bytes(n, Lp));
  L.tsqr = take(L.tsqr_bytes);
  if (host) {
    L.stage_bytes = (uint64_t)b * n * esz;
    for (int i = 0; i < 2; ++i) L.stage[i] = take(L.stage_bytes);
  }
  L.total = off;
  return L;
}

// Resolve the row block: the caller's value, or the largest that fits the budget.
int resolve_block(const brsvd_params& p, int64_t* b_out) {
  const bool host = p.a_location == BRSVD_A_HOST_PINNED;
  int64_t b = p.row_block > 0 ? std::min<int64_t>(p.row_block, p.m) : 0;
  uint64_t budget = p.device_budget_bytes;
  if (p.workspace) budget = budget ? std::min<uint64_t>(budget, p.workspace_bytes) : p.workspace_bytes;
  if (p.workspace && budget == 0) return BRSVD_ERR_BUDGET;
  if (b == 0) {
    if (!host) {
      b = p.m;
    } else {
      if (budget == 0) {
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) return BRSVD_ERR_HIP;
        budget = (uint64_t)(free_b * 0.8);
      }
      // largest multiple of 256 rows whose working set fits
      int64_t lo = 0, hi = (p.m + 255) / 256;
      while (lo < hi) {
        int64_t mid = (lo + hi + 1) / 2;
        int64_t bb = std::min<int64_t>(mid * 256, p.m);
        if (make_layout(p, bb).total <= budget) lo = mid; else hi = mid - 1;
      }
      if (lo == 0) return BRSVD_ERR_BUDGET;
      b = std::min<int64_t>(lo * 256, p.m);
    }
  }
  if ((p.device_budget_bytes || p.workspace) && make_layout(p, b).total > budget) return BRSVD_ERR_BUDGET;
  *b_out = b;
  return BRSVD_OK;
}

struct Region {
  brsvd_handle h;
  int cat;
  hipStream_t s;
  int i0;
  Region(brsvd_handle h_, int cat_, hipStream_t s_) : h(h_), cat(cat_), s(s_), i0(-1) {
    if (!h->timing || h->ev_used + 2 > h->ev.size()) return;
    // timing_level 1: only the pass kernels, the copies and the whole call are timed
    if (h->prm.timing_level == 1 && cat != CAT_TOTAL && cat != CAT_COPY && cat != CAT_UPD) return;
    i0 = (int)h->ev_used;
    h->ev_used += 2;
    (void)hipEventRecord(h->ev[i0], s);
  }
  ~Region() {
    if (i0 < 0) return;
    (void)hipEventRecord(h->ev[i0 + 1], s);
    h->regions[cat].push_back({i0, i0 + 1});
  }
};

// Accounts for one pass-kernel launch that reads `rows` rows of A, and hands out events from the pool
// for tight per-kernel timing: one pair registered under `cat`, one under CAT_SUM for the split sums.
bool kernel_events(brsvd_handle h, int cat, int64_t rows, KernelEvents* ke) {
  h->launches[cat]++;
  h->bytes_A_kernels += rows * h->prm.n * h->esz();
  if (!h->timing || h->ev_used + 4 > h->ev.size()) return false;
  int i0 = (int)h->ev_used;
  h->ev_used += 4;
  ke->start = h->ev[i0];
  ke->stop = h->ev[i0 + 1];
  ke->sum_start = h->ev[i0 + 2];
  ke->sum_stop = h->ev[i0 + 3];
  h->regions[cat].push_back({i0, i0 + 1});
  h->regions[CAT_SUM].push_back({i0 + 2, i0 + 3});
  return true;
}

template <typename T = float>
OrthWorkT<T> orth_work(brsvd_handle h) {
  OrthWorkT<T> w;
  w.gram_part = h->at<double>(h->lay.gram_part);
  w.gram_chunks_max = h->lay.gram_chunks;
  w.G = h->at<double>(h->lay.G);
  w.R[0] = h->at<double>(h->lay.R0);
  w.R[1] = h->at<double>(h->lay.R1);
  w.Xinv = h->at<double>(h->lay.Xinv);
  w.Rinv = h->at<T>(h->lay.Rinv);
  w.flags = h->at<int>(h->lay.flags);
  w.gemm_scratch = h->arena + h->lay.gemm_scratch;
  w.gemm_scratch_bytes = h->lay.gemm_scratch_bytes;
  w.tsqr_work = h->arena + h->lay.tsqr;
  w.tsqr_bytes = h->lay.tsqr_bytes;
  return w;
}

// ---- one pass over A ---------------------------------------------------------------------------
// Host-resident A: software pipeline over the two staging buffers.
struct Streamer {
  brsvd_handle h;
  const char* A;   // host-resident matrix, elements of h->esz() bytes
  int64_t lda;
  int issued;   // blocks whose copy has been enqueued in this pass
  Streamer(brsvd_handle h_, const void* A_, int64_t lda_) : h(h_), A((const char*)A_), lda(lda_), issued(0) {}
  int64_t rows_of(int i) const { return std::min<int64_t>(h->b, h->prm.m - (int64_t)i * h->b); }
  int enqueue_copy(int i) {
    const int buf = i & 1;
    // the buffer must have been consumed by the GEMM that last used it
    BRSVD_HIP_TRY(hipStreamWaitEvent(h->copy, h->drained[buf], 0));
    char* dst = h->at<char>(h->lay.stage[buf]);
    const size_t esz = (size_t)h->esz();
    const char* src = A + (int64_t)i * h->b * lda * esz;
    const int64_t rows = rows_of(i), n = h->prm.n;
    h->bytes_A_copied += rows * n * (int64_t)esz;
    Region r(h, CAT_COPY, h->copy);
    if (lda == n) {
      BRSVD_HIP_TRY(hipMemcpyAsync(dst, src, (size_t)rows * n * esz, hipMemcpyHostToDevice, h->copy));
    } else {
      BRSVD_HIP_TRY(hipMemcpy2DAsync(dst, (size_t)n * esz, src, (size_t)lda * esz, (size_t)n * esz, (size_t)rows,
                                     hipMemcpyHostToDevice, h->copy));
    }
    BRSVD_HIP_TRY(hipEventRecord(h->filled[buf], h->copy));
    return BRSVD_OK;
  }
  // make block i available to the compute stream; prefetch block i+1
  template <typename T>
  int acquire(int i, const T** blk) {
    if (issued == 0) { BRSVD_TRY(enqueue_copy(0)); issued = 1; }
    if (i + 1 < h->nblocks && issued == i + 1) { BRSVD_TRY(enqueue_copy(i + 1)); issued = i + 2; }
    BRSVD_HIP_TRY(hipStreamWaitEvent(h->compute, h->filled[i & 1], 0));
    *blk = h->at<T>(h->lay.stage[i & 1]);
    return BRSVD_OK;
  }
  int release(int i) {
    BRSVD_HIP_TRY(hipEventRecord(h->drained[i & 1], h->compute));
    return BRSVD_OK;
  }
};

template <typename T>
int pass_an(brsvd_handle h, const T* A, int64_t lda, const T* X, T* Y) {
  const int Lp = h->Lp;
  const int64_t m = h->prm.m, n = h->prm.n;
  void* scr = h->arena + h->lay.gemm_scratch;
  if (!h->host_a) {
    KernelEvents ke;
    bool t = kernel_events(h, CAT_AN, m, &ke);
    return gemm_an(A, lda, m, n, X, Lp, Y, Lp, Lp, scr, h->lay.gemm_scratch_bytes, h->compute, t ? &ke : nullptr);
  }
  Streamer st(h, A, lda);
  for (int i = 0; i < h->nblocks; ++i) {
    const T* blk;
    BRSVD_TRY(st.acquire(i, &blk));
    KernelEvents ke;
    bool t = kernel_events(h, CAT_AN, st.rows_of(i), &ke);
    BRSVD_TRY(gemm_an(blk, n, st.rows_of(i), n, X, Lp, Y + (int64_t)i * h->b * Lp, Lp, Lp, scr,
                      h->lay.gemm_scratch_bytes, h->compute, t ? &ke : nullptr));
    BRSVD_TRY(st.release(i));
  }
  return BRSVD_OK;
}

template <typename T>
int pass_at(brsvd_handle h, const T* A, int64_t lda, const T* Q, T* Z) {
  const int Lp = h->Lp;
  const int64_t m = h->prm.m, n = h->prm.n;
  void* scr = h->arena + h->lay.gemm_scratch;
  if (!h->host_a) {
    KernelEvents ke;
    bool t = kernel_events(h, CAT_AT, m, &ke);
    // device-resident A: one launch over all rows; the row range is cut into equal sub-ranges whose partial
    // panels are added in row order (the row blocks matter only when A is streamed block by block)
    return gemm_at(A, lda, m, n, Q, Lp, Z, false, m, scr, h->lay.gemm_scratch_bytes, h->compute,
                   t ? &ke : nullptr);
  }
  Streamer st(h, A, lda);
  for (int i = 0; i < h->nblocks; ++i) {
    const T* blk;
    BRSVD_TRY(st.acquire(i, &blk));
    KernelEvents ke;
    bool t = kernel_events(h, CAT_AT, st.rows_of(i), &ke);
    BRSVD_TRY(gemm_at(blk, n, st.rows_of(i), n, Q + (int64_t)i * h->b * Lp, Lp, Z, i > 0, st.rows_of(i), scr,
                      h->lay.gemm_scratch_bytes, h->compute, t ? &ke : nullptr));
    BRSVD_TRY(st.release(i));
  }
  return BRSVD_OK;
}

// One read of A doing both products of a power step: T_I = A_I * X and Z += A_I^T * T_I while block I
// is resident (device-resident A: two launches over the whole matrix).
template <typename T>
int pass_fused(brsvd_handle h, const T* A, int64_t lda, const T* X, T* Tm_, T* Z) {
  const int Lp = h->Lp;
  const int64_t n = h->prm.n;
  void* scr = h->arena + h->lay.gemm_scratch;
  if (!h->host_a) {
    BRSVD_TRY(pass_an<T>(h, A, lda, X, Tm_));
    return pass_at<T>(h, A, lda, Tm_, Z);
  }
  Streamer st(h, A, lda);
  for (int i = 0; i < h->nblocks; ++i) {
    const T* blk;
    BRSVD_TRY(st.acquire(i, &blk));
    T* Ti = Tm_ + (int64_t)i * h->b * Lp;
    KernelEvents ke;
    bool t = kernel_events(h, CAT_AN, st.rows_of(i), &ke);
    BRSVD_TRY(gemm_an(blk, n, st.rows_of(i), n, X, Lp, Ti, Lp, Lp, scr, h->lay.gemm_scratch_bytes, h->compute,
                      t ? &ke : nullptr));
    t = kernel_events(h, CAT_AT, st.rows_of(i), &ke);
    BRSVD_TRY(gemm_at(blk, n, st.rows_of(i), n, Ti, Lp, Z, i > 0, st.rows_of(i), scr, h->lay.gemm_scratch_bytes,
                      h->compute, t ? &ke : nullptr));
    BRSVD_TRY(st.release(i));
  }
  return BRSVD_OK;
}

// The whole factorisation, enqueued asynchronously on the handle's streams.
// Index (in doubles) into the handle's device scalars of the diagonal ratio of the factor of the sketch that a
// fused run leaves for the host (the slots before it belong to the robust-PCA loop and the power method).
constexpr int kScalFusedRatio = 7;

template <typename T>
int enqueue_brsvd(brsvd_handle h, const T* A, int64_t lda, const T* Omega, T* U, T* S, T* Vt, int method,
                  bool fused) {
  const int l = h->l, Lp = h->Lp, q = h->prm.q;
  const int64_t m = h->prm.m, n = h->prm.n;
  hipStream_t cs = h->compute;
  OrthWorkT<T> ow = orth_work<T>(h);
  void* scr = h->arena + h->lay.gemm_scratch;
  const uint64_t scr_bytes = h->lay.gemm_scratch_bytes;

  T* Xn = h->Pn<T>(0);    // current n x Lp panel (Omega, then W)
  T* Tn = h->Pn<T>(1);
  T* Ym = h->Pm<T>(0);    // current m x Lp panel
  T* Tm = h->Pm<T>(1);
  T* res;

  BRSVD_TRY(pad_panel(Omega, n, l, Xn, Lp, cs));
  if (fused) {
    // q passes Z = A^T (A X), X <- orth(Z), then one pass Y = A X, C^T = A^T Y; with Y = Q R the
    // projection is B^T = A^T Q = C^T R^-1, so R^-1 is applied to both panels.
    for (int it = 0; it < q; ++it) {
      BRSVD_TRY(pass_fused<T>(h, A, lda, Xn, Ym, Tn));
      Region r(h, CAT_ORTH, cs);
      BRSVD_TRY(orth_panel<T>(Tn, Xn, n, l, Lp, method, false, ow, nullptr, &res, cs));
      if (res != Xn) std::swap(Xn, Tn);
    }
    BRSVD_TRY(pass_fused<T>(h, A, lda, Xn, Ym, Tn));
    {
      Region r(h, CAT_ORTH, cs);
      ow.comp = Tn; ow.comp_tmp = Xn; ow.comp_rows = n;
      // the factor R of Y = Q R is kept (in the buffer the thin QR of B^T overwrites below) for its diagonal:
      // the host reads min |R_ii| / max |R_ii| at the end of the run and decides whether B^T = C^T R^-1 can be
      // trusted in this precision
      double* Ry = h->at<double>(h->lay.Rtot);
      BRSVD_TRY(orth_panel<T>(Ym, Tm, m, l, Lp, method, true, ow, Ry, &res, cs));
      BRSVD_TRY(diag_ratio(Ry, l, Lp, h->at<double>(h->lay.scal) + kScalFusedRatio, cs));
      if (res != Ym) std::swap(Ym, Tm);
      Xn = ow.comp; Tn = ow.comp_tmp;     // B^T and a free n x Lp buffer
      ow.comp = ow.comp_tmp = nullptr; ow.comp_rows = 0;
    }
  } else {
    BRSVD_TRY(pass_an<T>(h, A, lda, Xn, Ym));
    {
      Region r(h, CAT_ORTH, cs);
      BRSVD_TRY(orth_panel<T>(Ym, Tm, m, l, Lp, method, q == 0, ow, nullptr, &res, cs));
      if (res != Ym) std::swap(Ym, Tm);
    }
    for (int it = 0; it < q; ++it) {
      BRSVD_TRY(pass_at<T>(h, A, lda, Ym, Xn));
      {
        Region r(h, CAT_ORTH, cs);
        BRSVD_TRY(orth_panel<T>(Xn, Tn, n, l, Lp, method, false, ow, nullptr, &res, cs));
        if (res != Xn) std::swap(Xn, Tn);
      }
      BRSVD_TRY(pass_an<T>(h, A, lda, Xn, Tm));
      std::swap(Ym, Tm);
      {
        Region r(h, CAT_ORTH, cs);
        BRSVD_TRY(orth_panel<T>(Ym, Tm, m, l, Lp, method, it == q - 1, ow, nullptr, &res, cs));
        if (res != Ym) std::swap(Ym, Tm);
      }
    }
    // projection B^T = A^T Q
    BRSVD_TRY(pass_at<T>(h, A, lda, Ym, Xn));
  }
  // thin QR of B^T, the small SVD, the lifts
  double* Rtot = h->at<double>(h->lay.Rtot);
  {
    Region r(h, CAT_ORTH, cs);
    BRSVD_TRY(orth_panel<T>(Xn, Tn, n, l, Lp, method, true, ow, Rtot, &res, cs));
    if (res != Xn) std::swap(Xn, Tn);
  }
  SvdWork sw;
  sw.W = h->at<double>(h->lay.svdW);
  sw.J = h->at<double>(h->lay.svdJ);
  sw.sig = h->at<double>(h->lay.sig);
  sw.info = h->at<int>(h->lay.flags) + 4;
  T* XV = h->at<T>(h->lay.XV);
  T* XU = h->at<T>(h->lay.XU);
  {
    Region r(h, CAT_SVD, cs);
    BRSVD_TRY(small_svd<T>(Rtot, Lp, l, Lp, sw, ow.flags, nullptr, S, XV, XU, nullptr, nullptr, cs));
  }
  {
    Region r(h, CAT_LIFT, cs);
    BRSVD_TRY(gemm_an(Ym, Lp, m, Lp, XV, Lp, U, l, l, scr, scr_bytes, cs));          // U = Q * Vr
    BRSVD_TRY(gemm_an(Xn, Lp, n, Lp, XU, Lp, Tn, Lp, Lp, scr, scr_bytes, cs));       // V = W_B * Ur
    BRSVD_TRY(transpose_panel(Tn, n, Lp, l, Vt, cs));
  }
  return BRSVD_OK;
}

// The block-local scheme as Alg. 2 prints it, for a row-major A walked in row blocks (= column blocks of
// A^T, so the roles of m and n are those of the transposed problem):
//   first sweep    Y (n x l) += (A_I^T A_I)^q A_I^T Omega_I per resident block, factors applied right to
//                  left (Sec. 3 "Implementation details"); Omega_I is drawn on the device while the block is being copied
//   Q = orth(Y)
//   second sweep   C_I = A_I Q  (C = B^T, m x l)
//   C = W_C R, R = Ur diag(s) Vr^T   =>   A ~ (W_C Ur) diag(s) (Q Vr)^T
// Two reads of A whatever q is.  Omega (m x l, device) overrides the generator when not null.
template <typename T>
int enqueue_alg2(brsvd_handle h, const T* A, int64_t lda, uint64_t seed, const T* Omega, T* U, T* S, T* Vt,
                 int method) {
  const int l = h->l, Lp = h->Lp, q = h->prm.q;
  const int64_t m = h->prm.m, n = h->prm.n;
  hipStream_t cs = h->compute;
  OrthWorkT<T> ow = orth_work<T>(h);
  void* scr = h->arena + h->lay.gemm_scratch;
  const uint64_t scr_bytes = h->lay.gemm_scratch_bytes;
  T* Yn = h->Pn<T>(0);
  T* Pn1 = h->Pn<T>(1);
  T* OmI = h->Pm<T>(0);     // b x Lp windows of the two m x Lp panels
  T* TI = h->Pm<T>(1);
  T* res;

  Streamer st(h, A, lda);
  for (int i = 0; i < h->nblocks; ++i) {
    const int64_t rows = st.rows_of(i), r0 = (int64_t)i * h->b;
    if (Omega) BRSVD_TRY(pad_panel(Omega + r0 * l, rows, l, OmI, Lp, cs));
    else BRSVD_TRY(philox_normal<T>(seed, r0, rows, l, OmI, Lp, cs));
    const T* blk = A + r0 * lda;
    int64_t ldb = lda;
    if (h->host_a) { BRSVD_TRY(st.acquire(i, &blk)); ldb = n; }
    auto at = [&](const T* Qp, T* Z, bool accumulate) {
      KernelEvents ke;
      bool t = kernel_events(h, CAT_AT, rows, &ke);
      return gemm_at(blk, ldb, rows, n, Qp, Lp, Z, accumulate, rows, scr, scr_bytes, cs, t ? &ke : nullptr);
    };
    if (q == 0) {
      BRSVD_TRY(at(OmI, Yn, i > 0));
    } else {
      BRSVD_TRY(at(OmI, Pn1, false));
      for (int t = 0; t < q; ++t) {
        KernelEvents ke;
        bool tm = kernel_events(h, CAT_AN, rows, &ke);
        BRSVD_TRY(gemm_an(blk, ldb, rows, n, Pn1, Lp, TI, Lp, Lp, scr, scr_bytes, cs, tm ? &ke : nullptr));
        const bool last = t == q - 1;
        BRSVD_TRY(at(TI, last ? Yn : Pn1, last && i > 0));
      }
    }
    if (h->host_a) BRSVD_TRY(st.release(i));
  }
  {
    Region r(h, CAT_ORTH, cs);
    BRSVD_TRY(orth_panel<T>(Yn, Pn1, n, l, Lp, method, true, ow, nullptr, &res, cs));
    if (res != Yn) std::swap(Yn, Pn1);
  }
  T* Cm = h->Pm<T>(0);
  T* Tm = h->Pm<T>(1);
  BRSVD_TRY(pass_an<T>(h, A, lda, Yn, Cm));                 // second sweep: C = A Q
  double* Rtot = h->at<double>(h->lay.Rtot);
  {
    Region r(h, CAT_ORTH, cs);
    BRSVD_TRY(orth_panel<T>(Cm, Tm, m, l, Lp, method, true, ow, Rtot, &res, cs));
    if (res != Cm) std::swap(Cm, Tm);
  }
  SvdWork sw;
  sw.W = h->at<double>(h->lay.svdW);
  sw.J = h->at<double>(h->lay.svdJ);
  sw.sig = h->at<double>(h->lay.sig);
  sw.info = h->at<int>(h->lay.flags) + 4;
  T* XV = h->at<T>(h->lay.XV);
  T* XU = h->at<T>(h->lay.XU);
  {
    Region r(h, CAT_SVD, cs);
    BRSVD_TRY(small_svd<T>(Rtot, Lp, l, Lp, sw, ow.flags, nullptr, S, XV, XU, nullptr, nullptr, cs));
  }
  {
    Region r(h, CAT_LIFT, cs);
    BRSVD_TRY(gemm_an(Cm, Lp, m, Lp, XU, Lp, U, l, l, scr, scr_bytes, cs));            // U = W_C * Ur
    BRSVD_TRY(gemm_an(Yn, Lp, n, Lp, XV, Lp, Pn1, Lp, Lp, scr, scr_bytes, cs));        // V = Q * Vr
    BRSVD_TRY(transpose_panel(Pn1, n, Lp, l, Vt, cs));
  }
  return BRSVD_OK;
}

void reset_timing(brsvd_handle h, bool on) {
  h->timing = on;
  h->ev_used = 0;
  h->bytes_A_kernels = h->bytes_A_copied = 0;
  for (int c = 0; c < CAT_COUNT; ++c) { h->regions[c].clear(); h->launches[c] = 0; }
}

double sum_regions(brsvd_handle h, int cat) {
  double s = 0.0;
  for (auto& pr : h->regions[cat]) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, h->ev[pr.first], h->ev[pr.second]) == hipSuccess) s += ms * 1e-3;
  }
  return s;
}

// Reads of A are counted where they happen: a host-resident A is read over the host link by the block
// copies (the kernels then read the staged blocks), a device-resident A by the pass kernels themselves.
void fill_stats(brsvd_handle h, brsvd_stats* st, int fallbacks, int fused_fallbacks) {
  std::memset(st, 0, sizeof(*st));
  st->total_seconds = sum_regions(h, CAT_TOTAL);
  st->gemm_an_seconds = sum_regions(h, CAT_AN);
  st->gemm_at_seconds = sum_regions(h, CAT_AT);
  st->orth_seconds = sum_regions(h, CAT_ORTH);
  st->svd_seconds = sum_regions(h, CAT_SVD);
  st->lift_seconds = sum_regions(h, CAT_LIFT);
  st->copy_seconds = sum_regions(h, CAT_COPY);
  st->elementwise_seconds = sum_regions(h, CAT_ELEM);
  st->gemm_an_launches = h->launches[CAT_AN];
  st->gemm_at_launches = h->launches[CAT_AT];
  st->split_sum_seconds = sum_regions(h, CAT_SUM);
  st->rpca_update_seconds = sum_regions(h, CAT_UPD);
  st->rpca_update_launches = h->launches[CAT_UPD];
  st->bytes_A_streamed = h->host_a ? h->bytes_A_copied : h->bytes_A_kernels;
  st->bytes_A_read_by_kernels = h->bytes_A_kernels;
  st->passes_over_A = st->bytes_A_streamed / ((int64_t)h->esz() * h->prm.m * h->prm.n);
  st->orth_fallbacks = fallbacks;
  st->fused_fallbacks = fused_fallbacks;
  st->jacobi_sweeps = h->host_flags[1];
  st->row_block = (int32_t)h->b;
  st->n_blocks = h->nblocks;
}

void add_stats(brsvd_stats* acc, const brsvd_stats& s) {
  acc->total_seconds += s.total_seconds;
  acc->gemm_an_seconds += s.gemm_an_seconds;
  acc->gemm_at_seconds += s.gemm_at_seconds;
  acc->orth_seconds += s.orth_seconds;
  acc->svd_seconds += s.svd_seconds;
  acc->lift_seconds += s.lift_seconds;
  acc->copy_seconds += s.copy_seconds;
  acc->elementwise_seconds += s.elementwise_seconds;
  acc->split_sum_seconds += s.split_sum_seconds;
  acc->rpca_update_seconds += s.rpca_update_seconds;
  acc->rpca_update_launches += s.rpca_update_launches;
  acc->gemm_an_launches += s.gemm_an_launches;
  acc->gemm_at_launches += s.gemm_at_launches;
  acc->passes_over_A += s.passes_over_A;
  acc->bytes_A_streamed += s.bytes_A_streamed;
  acc->bytes_A_read_by_kernels += s.bytes_A_read_by_kernels;
  acc->orth_fallbacks += s.orth_fallbacks;
  acc->fused_fallbacks += s.fused_fallbacks;
  acc->jacobi_sweeps = s.jacobi_sweeps;
  acc->row_block = s.row_block;
  acc->n_blocks = s.n_blocks;
}

// Below this ratio min |R_ii| / max |R_ii| of the sketch's triangular factor the fused pass mode is not
// trusted: its projection B^T = C^T R^-1 amplifies the rounding noise of C^T (relative eps) by the square of
// the ratio's inverse, so once ratio^2 nears eps the trailing triplets are noise -- and noise that comes out
// LARGE, which would displace real singular values.  Measured in fp32 (k = 40, p = 10, q = 1, geometric
// spectra): sigma_l / sigma_1 = 1.7e-4 still gives 4e-5 relative accuracy, 8.7e-5 gives errors of order one.
inline double fused_ratio_floor(int dtype) { return dtype == BRSVD_DTYPE_F64 ? 3e-8 : 3e-4; }

// Runs one factorisation to completion (synchronises), handling two optimistic choices whose failure is
// only visible at the end: the CholeskyQR route (breakdown flag; AUTO then repeats the run with TSQR) and
// the fused pass mode (diagonal ratio of the sketch's factor below fused_ratio_floor: the run is repeated
// with separate passes, which re-orthonormalise after every product and have no such limit).
// enqueue(method, fused) queues one attempt; fused_possible = the caller asked for the fused mode.
template <typename Enqueue>
int run_sync_with(brsvd_handle h, bool fused_possible, int* fallbacks, int* fused_fallbacks, Enqueue enqueue) {
  int method = h->prm.orth_method;
  bool fused = fused_possible;
  int* dflags = h->at<int>(h->lay.flags);
  double* dratio = h->at<double>(h->lay.scal) + kScalFusedRatio;
  for (int attempt = 0; attempt < 3; ++attempt) {
    BRSVD_HIP_TRY(hipMemsetAsync(dflags, 0, 64, h->compute));
    if (h->host_a) {
      // the staging buffers start out free
      for (int i = 0; i < 2; ++i) BRSVD_HIP_TRY(hipEventRecord(h->drained[i], h->compute));
    }
    {
      // an error part-way leaves kernels and copies queued that still touch the caller's buffers and the
      // staging blocks: drain both streams before handing the status back
      const int st = enqueue(method, fused);
      if (st != BRSVD_OK) {
        (void)hipStreamSynchronize(h->compute);
        if (h->host_a) (void)hipStreamSynchronize(h->copy);
        return st;
      }
    }
    BRSVD_HIP_TRY(hipMemcpyAsync(h->host_flags, dflags, sizeof(int), hipMemcpyDeviceToHost, h->compute));
    BRSVD_HIP_TRY(hipMemcpyAsync(h->host_flags + 1, dflags + 4, 2 * sizeof(int), hipMemcpyDeviceToHost,
                                 h->compute));
    if (fused)
      BRSVD_HIP_TRY(hipMemcpyAsync(h->host_scal + kScalFusedRatio, dratio, sizeof(double), hipMemcpyDeviceToHost,
                                   h->compute));
    BRSVD_HIP_TRY(hipStreamSynchronize(h->compute));
    if (h->host_a) BRSVD_HIP_TRY(hipStreamSynchronize(h->copy));
    if (h->host_flags[0] != 0) {
      if (method != BRSVD_ORTH_AUTO) return BRSVD_ERR_ORTH_BREAKDOWN;
      method = BRSVD_ORTH_TSQR;
      if (fallbacks) ++*fallbacks;
      continue;
    }
    if (fused && !(h->host_scal[kScalFusedRatio] >= fused_ratio_floor(h->prm.dtype))) {
      fused = false;
      if (fused_fallbacks) ++*fused_fallbacks;
      continue;
    }
    if (h->host_flags[2] == 0) return BRSVD_ERR_SVD_NOCONV;
    return BRSVD_OK;
  }
  return BRSVD_ERR_ORTH_BREAKDOWN;
}

template <typename T>
int run_sync(brsvd_handle h, const T* A, int64_t lda, const T* Omega, T* U, T* S, T* Vt, int* fallbacks,
             int* fused_fallbacks) {
  return run_sync_with(h, h->prm.pass_mode == BRSVD_PASSES_FUSED, fallbacks, fused_fallbacks,
                       [&](int method, bool fused) { return enqueue_brsvd<T>(h, A, lda, Omega, U, S, Vt, method, fused); });
}

template <typename T>
int run_with_stats(brsvd_handle h, const T* A, int64_t lda, const T* Omega, T* U, T* S, T* Vt, brsvd_stats* stats) {
  if (!A || !Omega || !U || !S || !Vt) return BRSVD_ERR_ARG;
  if (lda < h->prm.n) return BRSVD_ERR_ARG;
  reset_timing(h, stats != nullptr);
  int fallbacks = 0, fused_fallbacks = 0, status;
  {
    Region total(h, CAT_TOTAL, h->compute);
    status = run_sync<T>(h, A, lda, Omega, U, S, Vt, &fallbacks, &fused_fallbacks);
  }
  if (stats) {
    (void)hipStreamSynchronize(h->compute);
    fill_stats(h, stats, fallbacks, fused_fallbacks);
  }
  return status;
}

template <typename T>
int run_alg2_with_stats(brsvd_handle h, const T* A, int64_t lda, uint64_t seed, const T* Omega, T* U, T* S, T* Vt,
                        brsvd_stats* stats) {
  if (!A || !U || !S || !Vt) return BRSVD_ERR_ARG;
  if (lda < h->prm.n) return BRSVD_ERR_ARG;
  reset_timing(h, stats != nullptr);
  int fallbacks = 0, status;
  {
    Region total(h, CAT_TOTAL, h->compute);
    status = run_sync_with(h, false, &fallbacks, nullptr, [&](int method, bool) {
      return enqueue_alg2<T>(h, A, lda, seed, Omega, U, S, Vt, method);
    });
  }
  if (stats) {
    (void)hipStreamSynchronize(h->compute);
    fill_stats(h, stats, fallbacks, 0);
  }
  return status;
}

// ---- power method for ||A||_2, both element types --------------------------------------------------
template <typename T>
int norm2_power_impl(brsvd_handle h, const T* A, int64_t lda, const T* x0, int32_t iters, double* norm2_out) {
  if (!A || !x0 || !norm2_out || iters < 1 || lda < h->prm.n || h->host_a) return BRSVD_ERR_ARG;
  const int64_t m = h->prm.m, n = h->prm.n;
  const int L1 = kTile;                 // the vector travels as column 0 of a 16-column padded panel
  hipStream_t cs = h->compute;
  T* xn = h->Pn<T>(0);
  T* zn = h->Pn<T>(1);
  T* ym = h->Pm<T>(0);
  void* scr = h->arena + h->lay.gemm_scratch;
  const uint64_t scr_bytes = h->lay.gemm_scratch_bytes;
  double* part = h->at<double>(h->lay.rpca_part);
  double* scal = h->at<double>(h->lay.scal);
  BRSVD_TRY(pad_panel(x0, n, 1, xn, L1, cs));
  BRSVD_TRY(rpca_norms<T>(xn, n * L1, part, scal, cs));
  BRSVD_TRY(scale_rsqrt<T>(xn, n * L1, scal + 1, cs));
  for (int it = 0; it < iters; ++it) {
    BRSVD_TRY(gemm_an(A, lda, m, n, xn, L1, ym, L1, L1, scr, scr_bytes, cs));              // y = A x
    BRSVD_TRY(rpca_norms<T>(ym, m * L1, part, scal + 2, cs));                                  // est^2 = |y|^2
    BRSVD_TRY(gemm_at(A, lda, m, n, ym, L1, zn, false, m, scr, scr_bytes, cs));            // z = A^T y
    BRSVD_TRY(rpca_norms<T>(zn, n * L1, part, scal + 4, cs));
    BRSVD_TRY(scale_rsqrt<T>(zn, n * L1, scal + 5, cs));                                       // x = z / |z|
    std::swap(xn, zn);
  }
  BRSVD_HIP_TRY(hipMemcpyAsync(h->host_scal, scal + 3, sizeof(double), hipMemcpyDeviceToHost, cs));
  BRSVD_HIP_TRY(hipStreamSynchronize(cs));
  *norm2_out = std::sqrt(h->host_scal[0]);
  return BRSVD_OK;
}


// ---- robust PCA loop (Alg. 3), both element types -----------------------------------------------
template <typename T>
int rpca_loop(brsvd_handle h, const T* M, const T* Omegas, int32_t max_iters, double tol, double lambda, double mu0,
              double rho, double norm2_M, T* L, T* S, T* work, double* residuals, int32_t* iters_done,
              brsvd_stats* stats) {
  if (iters_done) *iters_done = 0;
  if (!h || !M || !Omegas || !L || !S || !work || max_iters < 1) return BRSVD_ERR_ARG;
  if (h->host_a || !(lambda > 0.0) || !(mu0 > 0.0) || !(rho > 1.0) || !(tol >= 0.0)) return BRSVD_ERR_ARG;
  const int64_t m = h->prm.m, n = h->prm.n, count = m * n;
  const int l = h->l;
  hipStream_t cs = h->compute;
  // The multiplier alternates between the first half of `work` and L (an output nobody reads before the loop ends),
  // so the multiplier an iteration read is still there when the loop stops and L and S are formed from it.
  T* Ycur = work;
  T* Yalt = L;
  T* X = work + count;
  T* Uw = h->at<T>(h->lay.rpcaU);
  T* Vtw = h->at<T>(h->lay.rpcaVt);
  T* Sw = h->at<T>(h->lay.S32);
  double* part = h->at<double>(h->lay.rpca_part);
  double* scal = h->at<double>(h->lay.scal);
  brsvd_stats acc;
  std::memset(&acc, 0, sizeof(acc));
  auto flush_stats = [&](int fallbacks, int fused_fallbacks) {
    if (!stats) return;
    (void)hipStreamSynchronize(cs);
    brsvd_stats one;
    fill_stats(h, &one, fallbacks, fused_fallbacks);
    add_stats(&acc, one);
    reset_timing(h, true);
  };
  reset_timing(h, stats != nullptr);

  // ||M||_max, ||M||_F^2 and, if not supplied, ||M||_2 from one randomized SVD
  {
    Region r(h, CAT_ELEM, cs);
    BRSVD_TRY(rpca_norms<T>(M, count, part, scal, cs));
  }
  BRSVD_HIP_TRY(hipMemcpyAsync(h->host_scal, scal, 2 * sizeof(double), hipMemcpyDeviceToHost, cs));
  BRSVD_HIP_TRY(hipStreamSynchronize(cs));
  const double max_abs = h->host_scal[0], normF = std::sqrt(h->host_scal[1]);
  if (!(normF > 0.0)) return BRSVD_ERR_ARG;
  if (!(norm2_M > 0.0)) {
    int fb = 0, ffb = 0;
    {
      Region total(h, CAT_TOTAL, cs);
      BRSVD_TRY(run_sync<T>(h, M, n, Omegas, Uw, Sw, Vtw, &fb, &ffb));
    }
    T s0 = T(0);
    BRSVD_HIP_TRY(hipMemcpy(&s0, Sw, sizeof(T), hipMemcpyDeviceToHost));
    norm2_M = (double)s0;
    flush_stats(fb, ffb);
    if (!(norm2_M > 0.0)) return BRSVD_ERR_ARG;
  }
  const double J = std::max(norm2_M, max_abs / (double)lambda);
  double mu = mu0;
  {
    Region r(h, CAT_ELEM, cs);
    BRSVD_TRY(rpca_init<T>(M, count, (T)(1.0 / J), (T)(1.0 / mu), Ycur, S, X, cs));
  }
  int it = 0;
  double mu_last = mu;
  while (it < max_iters) {
    int fb = 0, ffb = 0;
    const double mu_next = mu * (double)rho;
    mu_last = mu;
    {
      Region total(h, CAT_TOTAL, cs);
      BRSVD_TRY(run_sync<T>(h, X, n, Omegas + (int64_t)it * n * l, Uw, Sw, Vtw, &fb, &ffb));
      {
        Region r(h, CAT_ELEM, cs);
        int nparts = 0;
        {
          Region u(h, CAT_UPD, cs);
          h->launches[CAT_UPD]++;
          BRSVD_TRY(rpca_update<T>(M, Uw, Sw, Vtw, m, n, l, (T)mu, (T)lambda, (T)mu_next, Ycur, Yalt, X, part, &nparts,
                                   cs));
          std::swap(Ycur, Yalt);                       // Yalt: what this iteration read
        }
        BRSVD_TRY(rpca_residual_sum(part, nparts, scal + 2, cs));
      }
      BRSVD_HIP_TRY(hipMemcpyAsync(h->host_scal + 2, scal + 2, sizeof(double), hipMemcpyDeviceToHost, cs));
      BRSVD_HIP_TRY(hipStreamSynchronize(cs));
    }
    const double res = std::sqrt(h->host_scal[2]) / normF;
    if (residuals) residuals[it] = res;
    flush_stats(fb, ffb);
    ++it;
    if (res < tol) break;       // the stopping rule of Alg. 3: mu is not advanced any more
    mu = mu_next;
  }
  // L and S of the last iteration run: its triplets, its mu and the multiplier it read are still in place
  {
    Region r(h, CAT_ELEM, cs);
    BRSVD_TRY(rpca_finalize<T>(M, Uw, Sw, Vtw, m, n, l, (T)mu_last, (T)lambda, Yalt, L, S, cs));
  }
  BRSVD_HIP_TRY(hipStreamSynchronize(cs));
  flush_stats(0, 0);
  if (iters_done) *iters_done = it;
  if (stats) *stats = acc;
  return BRSVD_OK;
}


// ---- step-level GEMM calls (both element types) --------------------------------------------------
uint64_t step_gemm_scratch_bytes(int64_t rows, int64_t n, int l, int esz) {
  if (rows < 1 || n < 1 || l < 1 || l > kMaxL) return 0;
  const int Lp = padded_l(l);
  const uint64_t panel = align_up((uint64_t)std::max(rows, n) * Lp * esz);
  uint64_t part = std::max(gemm_an_scratch_bytes(rows, n, Lp, esz), gemm_at_scratch_bytes(rows, n, Lp, rows, esz));
  return 2 * panel + align_up(part);
}

template <typename T>
int step_gemm_an(const T* A, int64_t lda, int64_t rows, int64_t n, const T* X, int l, T* Y, void* scratch,
                 uint64_t scratch_bytes, void* stream) {
  if (!A || !X || !Y || rows < 1 || n < 1 || l < 1 || l > kMaxL || lda < n) return BRSVD_ERR_ARG;
  if (!scratch || scratch_bytes < step_gemm_scratch_bytes(rows, n, l, (int)sizeof(T))) return BRSVD_ERR_BUDGET;
  const int Lp = padded_l(l);
  const uint64_t panel = align_up((uint64_t)std::max(rows, n) * Lp * sizeof(T));
  T* Xp = (T*)scratch;
  char* part = (char*)scratch + 2 * panel;
  hipStream_t s = (hipStream_t)stream;
  BRSVD_TRY(pad_panel(X, n, l, Xp, Lp, s));
  return gemm_an(A, lda, rows, n, Xp, Lp, Y, l, l, part, scratch_bytes - 2 * panel, s);
}

template <typename T>
int step_gemm_at(const T* A, int64_t lda, int64_t rows, int64_t n, const T* Q, int l, T* Z, int accumulate,
                 void* scratch, uint64_t scratch_bytes, void* stream) {
  if (!A || !Q || !Z || rows < 1 || n < 1 || l < 1 || l > kMaxL || lda < n) return BRSVD_ERR_ARG;
  if (!scratch || scratch_bytes < step_gemm_scratch_bytes(rows, n, l, (int)sizeof(T))) return BRSVD_ERR_BUDGET;
  const int Lp = padded_l(l);
  const uint64_t panel = align_up((uint64_t)std::max(rows, n) * Lp * sizeof(T));
  T* Qp = (T*)scratch;
  T* Zp = (T*)((char*)scratch + panel);
  char* part = (char*)scratch + 2 * panel;
  hipStream_t s = (hipStream_t)stream;
  BRSVD_TRY(pad_panel(Q, rows, l, Qp, Lp, s));
  BRSVD_TRY(gemm_at(A, lda, rows, n, Qp, Lp, Zp, false, rows, part, scratch_bytes - 2 * panel, s));
  return unpad_panel(Zp, n, Lp, l, Z, accumulate != 0, s);
}

// ---- small SVD on a given scratch buffer ---------------------------------------------------------
// Scratch of small_svd: the rows being rotated and one more Lp x Lp fp64 matrix, 3*Lp doubles (norms,
// sorted values, order) and a few integer flags.  Nothing in it has to be initialised: every kernel
// writes what it later reads.
constexpr uint64_t small_svd_scratch_bytes(int Lp) {
  return 2 * align_up((uint64_t)Lp * Lp * 8) + align_up((uint64_t)3 * Lp * 8) + 256;
}

int small_svd_on_scratch(const double* R, int l, double* S, double* Ur, double* Vr, int32_t* sweeps, char* buf,
                         hipStream_t s) {
  const int Lp = padded_l(l);
  const uint64_t sq8 = align_up((uint64_t)Lp * Lp * 8);
  SvdWork w;
  w.W = (double*)buf;
  w.J = (double*)(buf + sq8);
  w.sig = (double*)(buf + 2 * sq8);
  w.info = (int*)(buf + 2 * sq8 + align_up((uint64_t)3 * Lp * 8));
  int status = small_svd<float>(R, l, l, Lp, w, nullptr, S, nullptr, nullptr, nullptr, Ur, Vr, s);
  int info[2] = {0, 0};
  if (status == BRSVD_OK) {
    if (hipMemcpyAsync(info, w.info, sizeof(info), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      status = BRSVD_ERR_HIP;
  }
  (void)hipStreamSynchronize(s);
  if (status == BRSVD_OK) {
    if (sweeps) *sweeps = info[0];
    if (!info[1]) status = BRSVD_ERR_SVD_NOCONV;
  }
  return status;
}

// Scratch of brsvd_small_svd_static: a device array that is part of the loaded code object, so callers
// that may not allocate device memory can still run the small SVD.  Every GPU the library runs on holds
// its own copy (4.0 MiB) at its own address until the process ends.  `scratch` is only the host-side name
// of the symbol: the device address is looked up once per device and kept in g_static_scratch.
constexpr int kStaticSvdMaxL = 512;
constexpr uint64_t kStaticScratchBytes = small_svd_scratch_bytes(kStaticSvdMaxL);

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_scratch_mutex;
char* g_static_scratch[kMaxDevices];

int static_scratch_of_current_device(char** out) {
  int dev = -1;
  BRSVD_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return BRSVD_ERR_ARG;
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    BRSVD_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return BRSVD_ERR_HIP;
    g_static_scratch[dev] = (char*)p;
  }
  *out = g_static_scratch[dev];
  return BRSVD_OK;
}

}  // namespace

// ================================================================================================
// C ABI
// ================================================================================================
extern "C" {

int brsvd_workspace_bytes(const brsvd_params* params, uint64_t* bytes_out) {
  if (!bytes_out) return BRSVD_ERR_ARG;
  BRSVD_TRY(validate(params));
  int64_t b;
  BRSVD_TRY(resolve_block(*params, &b));
  *bytes_out = make_layout(*params, b).total;
  return BRSVD_OK;
}

static int create_impl(const brsvd_params* params, brsvd_handle* handle_out) {
  BRSVD_TRY(validate(params));
  int64_t b;
  BRSVD_TRY(resolve_block(*params, &b));
  brsvd_handle h = new (std::nothrow) brsvd_handle_s();
  if (!h) return BRSVD_ERR_ALLOC;
  h->prm = *params;
  h->l = params->k + params->p;
  h->Lp = padded_l(h->l);
  h->b = b;
  h->nblocks = (int)ceil_div(params->m, b);
  h->host_a = params->a_location == BRSVD_A_HOST_PINNED;
  h->lay = make_layout(*params, b);
  h->arena = nullptr;
  h->compute = (hipStream_t)params->compute_stream;
  h->copy = (hipStream_t)params->copy_stream;
  h->own_copy = false;
  h->host_flags = nullptr;
  h->host_scal = nullptr;
  h->ev_used = 0;
  h->timing = false;
  h->own_arena = params->workspace == nullptr;
  for (int i = 0; i < 2; ++i) { h->filled[i] = nullptr; h->drained[i] = nullptr; }
  int status = BRSVD_OK;
  do {
    if (h->own_arena) {
      if (hipMalloc((void**)&h->arena, h->lay.total) != hipSuccess) { status = BRSVD_ERR_ALLOC; break; }
    } else {
      h->arena = (char*)params->workspace;      // resolve_block has checked that it is large enough
    }
    if (hipMemset(h->arena + h->lay.gram_part, 0, (size_t)h->lay.gram_chunks * h->Lp * h->Lp * 8) != hipSuccess) {
      status = BRSVD_ERR_HIP; break;
    }
    if (hipHostMalloc((void**)&h->host_flags, 64, hipHostMallocDefault) != hipSuccess) { status = BRSVD_ERR_ALLOC; break; }
    if (hipHostMalloc((void**)&h->host_scal, 64, hipHostMallocDefault) != hipSuccess) { status = BRSVD_ERR_ALLOC; break; }
    std::memset(h->host_flags, 0, 64);
    if (h->host_a) {
      if (!h->copy) {
        if (hipStreamCreateWithFlags(&h->copy, hipStreamNonBlocking) != hipSuccess) { status = BRSVD_ERR_HIP; break; }
        h->own_copy = true;
      }
      bool ok = true;
      for (int i = 0; i < 2 && ok; ++i) {
        ok = hipEventCreateWithFlags(&h->filled[i], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&h->drained[i], hipEventDisableTiming) == hipSuccess;
      }
      if (!ok) { status = BRSVD_ERR_HIP; break; }
    }
    // per block and pass at most two products (4 events each) and one copy (2 events)
    const size_t pool = 64 + (size_t)h->nblocks * 12 * (2 * params->q + 2);
    try {
      h->ev.resize(pool, nullptr);
      for (int c = 0; c < CAT_COUNT; ++c) h->regions[c].reserve(pool / 2);   // no growth while a run records
    } catch (...) { status = BRSVD_ERR_ALLOC; break; }
    bool ok = true;
    for (size_t i = 0; i < pool && ok; ++i) ok = hipEventCreate(&h->ev[i]) == hipSuccess;
    if (!ok) { status = BRSVD_ERR_HIP; break; }
  } while (0);
  if (status != BRSVD_OK) {
    brsvd_destroy(h);
    return status;
  }
  *handle_out = h;
  return BRSVD_OK;
}

int brsvd_create(const brsvd_params* params, brsvd_handle* handle_out) {
  if (!handle_out) return BRSVD_ERR_ARG;
  *handle_out = nullptr;
  try {
    return create_impl(params, handle_out);
  } catch (...) {            // nothing may propagate across the C boundary
    return BRSVD_ERR_ALLOC;
  }
}

int brsvd_destroy(brsvd_handle h) {
  if (!h) return BRSVD_OK;
  if (h->arena) (void)hipDeviceSynchronize();
  for (auto e : h->ev) if (e) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; ++i) {
    if (h->filled[i]) (void)hipEventDestroy(h->filled[i]);
    if (h->drained[i]) (void)hipEventDestroy(h->drained[i]);
  }
  if (h->own_copy && h->copy) (void)hipStreamDestroy(h->copy);
  if (h->host_flags) (void)hipHostFree(h->host_flags);
  if (h->host_scal) (void)hipHostFree(h->host_scal);
  if (h->arena && h->own_arena) (void)hipFree(h->arena);
  delete h;
  return BRSVD_OK;
}

int brsvd_run(brsvd_handle h, const float* A, int64_t lda, const float* Omega, float* U, float* S, float* Vt,
              brsvd_stats* stats) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F32) return BRSVD_ERR_ARG;
  return run_with_stats<float>(h, A, lda, Omega, U, S, Vt, stats);
}

int brsvd_run_f64(brsvd_handle h, const double* A, int64_t lda, const double* Omega, double* U, double* S,
                  double* Vt, brsvd_stats* stats) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  return run_with_stats<double>(h, A, lda, Omega, U, S, Vt, stats);
}

int brsvd_run_alg2(brsvd_handle h, const float* A, int64_t lda, uint64_t seed, const float* Omega, float* U,
                   float* S, float* Vt, brsvd_stats* stats) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F32) return BRSVD_ERR_ARG;
  return run_alg2_with_stats<float>(h, A, lda, seed, Omega, U, S, Vt, stats);
}

int brsvd_run_alg2_f64(brsvd_handle h, const double* A, int64_t lda, uint64_t seed, const double* Omega, double* U,
                       double* S, double* Vt, brsvd_stats* stats) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  return run_alg2_with_stats<double>(h, A, lda, seed, Omega, U, S, Vt, stats);
}

int brsvd_gemm_plan(int32_t which, int64_t rows, int64_t n, int32_t l, int64_t block_rows, int32_t dtype,
                    int32_t* out12) {
  if (!out12 || rows < 1 || n < 1 || l < 1 || l > kMaxL) return BRSVD_ERR_ARG;
  if (dtype != BRSVD_DTYPE_F32 && dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  const int esz = dtype == BRSVD_DTYPE_F64 ? 8 : 4;
  if (which == 0) gemm_an_plan_describe(rows, n, padded_l(l), esz, out12);
  else if (which == 1) gemm_at_plan_describe(rows, n, padded_l(l), block_rows, esz, out12);
  else if (which == 2) {
    const uint64_t an = gemm_an_scratch_bytes(rows, n, padded_l(l), esz);
    const uint64_t at = gemm_at_scratch_bytes(rows, n, padded_l(l), block_rows, esz);
    for (int i = 0; i < 12; ++i) out12[i] = 0;
    out12[0] = (int32_t)(an & 0x7fffffff); out12[1] = (int32_t)(an >> 31);
    out12[2] = (int32_t)(at & 0x7fffffff); out12[3] = (int32_t)(at >> 31);
  } else return BRSVD_ERR_ARG;
  return BRSVD_OK;
}

int brsvd_probe(int32_t kind, void* buf, uint64_t amount, double* seconds, double* work, void* stream) {
  return probe(kind, buf, amount, seconds, work, (hipStream_t)stream);
}

int brsvd_philox_normal(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, float* out, void* stream) {
  if (!out || rows < 1 || cols < 1 || row0 < 0) return BRSVD_ERR_ARG;
  return philox_normal<float>(seed, row0, rows, cols, out, cols, (hipStream_t)stream);
}

int brsvd_philox_normal_f64(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, double* out, void* stream) {
  if (!out || rows < 1 || cols < 1 || row0 < 0) return BRSVD_ERR_ARG;
  return philox_normal<double>(seed, row0, rows, cols, out, cols, (hipStream_t)stream);
}

int brsvd_rpca_ialm_tol(brsvd_handle h, const float* M, const float* Omegas, int32_t max_iters, double tol,
                        float lambda, float mu0, float rho, double norm2_M, float* L, float* S, float* work,
                        double* residuals, int32_t* iters_done, brsvd_stats* stats) {
  if (iters_done) *iters_done = 0;
  if (!h || h->prm.dtype != BRSVD_DTYPE_F32) return BRSVD_ERR_ARG;
  return rpca_loop<float>(h, M, Omegas, max_iters, tol, lambda, mu0, rho, norm2_M, L, S, work, residuals, iters_done,
                          stats);
}

int brsvd_rpca_ialm_tol_f64(brsvd_handle h, const double* M, const double* Omegas, int32_t max_iters, double tol,
                            double lambda, double mu0, double rho, double norm2_M, double* L, double* S, double* work,
                            double* residuals, int32_t* iters_done, brsvd_stats* stats) {
  if (iters_done) *iters_done = 0;
  if (!h || h->prm.dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  return rpca_loop<double>(h, M, Omegas, max_iters, tol, lambda, mu0, rho, norm2_M, L, S, work, residuals, iters_done,
                           stats);
}

int brsvd_rpca_ialm(brsvd_handle h, const float* M, const float* Omegas, int32_t iters, float lambda, float mu0,
                    float rho, double norm2_M, float* L, float* S, float* work, double* residuals,
                    brsvd_stats* stats) {
  return brsvd_rpca_ialm_tol(h, M, Omegas, iters, 0.0, lambda, mu0, rho, norm2_M, L, S, work, residuals, nullptr,
                             stats);
}

int brsvd_norm2_power(brsvd_handle h, const float* A, int64_t lda, const float* x0, int32_t iters,
                      double* norm2_out) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F32) return BRSVD_ERR_ARG;
  return norm2_power_impl<float>(h, A, lda, x0, iters, norm2_out);
}

int brsvd_norm2_power_f64(brsvd_handle h, const double* A, int64_t lda, const double* x0, int32_t iters,
                          double* norm2_out) {
  if (!h || h->prm.dtype != BRSVD_DTYPE_F64) return BRSVD_ERR_ARG;
  return norm2_power_impl<double>(h, A, lda, x0, iters, norm2_out);
}

const char* brsvd_status_string(int status) {
  switch (status) {
    case BRSVD_OK: return "ok";
    case BRSVD_ERR_ARG: return "invalid argument";
    case BRSVD_ERR_BUDGET: return "device memory budget or scratch too small for the working set";
    case BRSVD_ERR_ALLOC: return "memory allocation failed";
    case BRSVD_ERR_HIP: return "HIP runtime error";
    case BRSVD_ERR_ORTH_BREAKDOWN: return "panel orthonormalisation broke down (numerically rank deficient)";
    case BRSVD_ERR_SVD_NOCONV: return "Jacobi SVD did not converge";
    default: return "unknown status";
  }
}

// ---- step-level entry points --------------------------------------------------------------------

uint64_t brsvd_gemm_scratch_bytes(int64_t rows, int64_t n, int32_t l) { return step_gemm_scratch_bytes(rows, n, l, 4); }
uint64_t brsvd_gemm_scratch_bytes_f64(int64_t rows, int64_t n, int32_t l) { return step_gemm_scratch_bytes(rows, n, l, 8); }

int brsvd_gemm_an(const float* A, int64_t lda, int64_t rows, int64_t n, const float* X, int32_t l, float* Y,
                  void* scratch, uint64_t scratch_bytes, void* stream) {
  return step_gemm_an<float>(A, lda, rows, n, X, l, Y, scratch, scratch_bytes, stream);
}
int brsvd_gemm_an_f64(const double* A, int64_t lda, int64_t rows, int64_t n, const double* X, int32_t l, double* Y,
                      void* scratch, uint64_t scratch_bytes, void* stream) {
  return step_gemm_an<double>(A, lda, rows, n, X, l, Y, scratch, scratch_bytes, stream);
}
int brsvd_gemm_at(const float* A, int64_t lda, int64_t rows, int64_t n, const float* Q, int32_t l, float* Z,
                  int32_t accumulate, void* scratch, uint64_t scratch_bytes, void* stream) {
  return step_gemm_at<float>(A, lda, rows, n, Q, l, Z, accumulate, scratch, scratch_bytes, stream);
}
int brsvd_gemm_at_f64(const double* A, int64_t lda, int64_t rows, int64_t n, const double* Q, int32_t l, double* Z,
                      int32_t accumulate, void* scratch, uint64_t scratch_bytes, void* stream) {
  return step_gemm_at<double>(A, lda, rows, n, Q, l, Z, accumulate, scratch, scratch_bytes, stream);
}

// Scratch of brsvd_orth: two padded panels, the Gram partial sums, five l x l fp64 factors, the inverse
// factor in the panels' type, flags, the split-sum scratch of the apply product and the TSQR work area.
struct OrthScratch {
  uint64_t panel, sq8, sq4, gs, tb, total;
  int chunks;
};
static OrthScratch orth_scratch_layout(int64_t rows, int Lp) {
  OrthScratch o;
  o.panel = align_up((uint64_t)rows * Lp * 4);
  o.sq8 = align_up((uint64_t)Lp * Lp * 8);
  o.sq4 = align_up((uint64_t)Lp * Lp * 4);
  o.chunks = (int)orth_gram_slots(rows, Lp);
  o.gs = align_up(gemm_an_scratch_bytes(rows, Lp, Lp));
  o.tb = align_up(tsqr_work_bytes(rows, Lp));
  o.total = 2 * o.panel + (uint64_t)o.chunks * o.sq8 + 5 * o.sq8 + o.sq4 + 256 + o.gs + o.tb;
  return o;
}

uint64_t brsvd_orth_scratch_bytes(int64_t rows, int32_t l) {
  if (rows < 1 || l < 1 || l > kMaxL) return 0;
  return orth_scratch_layout(rows, padded_l(l)).total;
}

int brsvd_orth(float* P, int64_t rows, int32_t l, int32_t method, double* R, int32_t* fallback_taken,
               void* scratch, uint64_t scratch_bytes, void* stream) {
  if (!P || rows < 1 || l < 1 || l > kMaxL || rows < l) return BRSVD_ERR_ARG;
  if (method < BRSVD_ORTH_AUTO || method > BRSVD_ORTH_TSQR) return BRSVD_ERR_ARG;
  if (!scratch || ((uintptr_t)scratch) % kAlign != 0) return BRSVD_ERR_ARG;
  if (fallback_taken) *fallback_taken = 0;
  const int Lp = padded_l(l);
  hipStream_t s = (hipStream_t)stream;
  const OrthScratch o = orth_scratch_layout(rows, Lp);
  if (scratch_bytes < o.total) return BRSVD_ERR_BUDGET;
  char* buf = (char*)scratch;
  int status = BRSVD_OK;
  do {
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { char* p = buf + off; off += bytes; return p; };
    float* P0 = (float*)take(o.panel);
    float* P1 = (float*)take(o.panel);
    OrthWork w;
    w.gram_part = (double*)take((uint64_t)o.chunks * o.sq8);
    w.gram_chunks_max = o.chunks;
    w.G = (double*)take(o.sq8); w.R[0] = (double*)take(o.sq8); w.R[1] = (double*)take(o.sq8);
    w.Xinv = (double*)take(o.sq8);
    double* Rtot = (double*)take(o.sq8);
    w.Rinv = (float*)take(o.sq4);
    w.flags = (int*)take(256);
    w.gemm_scratch = take(o.gs); w.gemm_scratch_bytes = o.gs;
    w.tsqr_work = take(o.tb); w.tsqr_bytes = o.tb;
    if (hipMemsetAsync(buf, 0, o.total, s) != hipSuccess) { status = BRSVD_ERR_HIP; break; }
    int m_now = method;
    for (int attempt = 0; attempt < 2; ++attempt) {
      float* res = nullptr;
      if ((status = pad_panel(P, rows, l, P0, Lp, s)) != BRSVD_OK) break;
      if (hipMemsetAsync(w.flags, 0, 256, s) != hipSuccess) { status = BRSVD_ERR_HIP; break; }
      if ((status = orth_panel(P0, P1, rows, l, Lp, m_now, true, w, Rtot, &res, s)) != BRSVD_OK) break;
      int flag = 0;
      if (hipMemcpyAsync(&flag, w.flags, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
          hipStreamSynchronize(s) != hipSuccess) { status = BRSVD_ERR_HIP; break; }
      if (flag == 0) {
        if ((status = unpad_panel(res, rows, Lp, l, P, false, s)) != BRSVD_OK) break;
        if (R) {
          if (hipMemcpy2DAsync(R, (size_t)l * 8, Rtot, (size_t)Lp * 8, (size_t)l * 8, (size_t)l,
                               hipMemcpyDeviceToDevice, s) != hipSuccess) { status = BRSVD_ERR_HIP; break; }
        }
        if (hipStreamSynchronize(s) != hipSuccess) status = BRSVD_ERR_HIP;
        break;
      }
      if (m_now != BRSVD_ORTH_AUTO) { status = BRSVD_ERR_ORTH_BREAKDOWN; break; }
      m_now = BRSVD_ORTH_TSQR;
      if (fallback_taken) *fallback_taken = 1;
    }
  } while (0);
  (void)hipStreamSynchronize(s);
  return status;
}

uint64_t brsvd_small_svd_scratch_bytes(int32_t l) {
  if (l < 1 || l > kMaxL) return 0;
  return small_svd_scratch_bytes(padded_l(l));
}

int brsvd_small_svd(const double* R, int32_t l, double* S, double* Ur, double* Vr, int32_t* sweeps, void* scratch,
                    uint64_t scratch_bytes, void* stream) {
  if (!R || !S || !Ur || !Vr || l < 1 || l > kMaxL) return BRSVD_ERR_ARG;
  if (!scratch || ((uintptr_t)scratch) % kAlign != 0) return BRSVD_ERR_ARG;
  if (scratch_bytes < small_svd_scratch_bytes(padded_l(l))) return BRSVD_ERR_BUDGET;
  return small_svd_on_scratch(R, l, S, Ur, Vr, sweeps, (char*)scratch, (hipStream_t)stream);
}

int brsvd_small_svd_static(const double* R, int32_t l, double* S, double* Ur, double* Vr, int32_t* sweeps,
                           void* stream) {
  if (!R || !S || !Ur || !Vr || l < 1) return BRSVD_ERR_ARG;
  if (l > kStaticSvdMaxL) return BRSVD_ERR_BUDGET;        // beyond what the static array was sized for
  char* buf = nullptr;
  BRSVD_TRY(static_scratch_of_current_device(&buf));
  return small_svd_on_scratch(R, l, S, Ur, Vr, sweeps, buf, (hipStream_t)stream);
}

}  // extern "C"
