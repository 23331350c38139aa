/*
 * brsvd.h -- C ABI of the MI355X (gfx950) block randomized SVD library.
 *
 * The library computes the rank-l (l = k + p) randomized SVD of an m x n fp32 matrix A
 * by the two-stage scheme of Alg. 1 of the paper (sketch Y = A*Omega, q power iterations
 * with A*A^T, orthonormal basis Q, projection B = Q^T*A, small SVD of B, lift U = Q*Ut),
 * with A visited one row block at a time and only the thin panels (m x l, n x l) kept on
 * the device, as in the block method of Alg. 2 / Sec. 3.  A may live in device memory or in
 * pinned host memory; in the latter case row blocks are streamed through two staging
 * buffers on a copy stream while the previous block is being multiplied.
 *
 * All matrices are ROW-MAJOR.  All entry points return an int status (0 = success,
 * negative = error), never throw, and never abort.  The library is not re-entrant per
 * handle: one brsvd_run / brsvd_rpca_ialm at a time per handle.
 */
#ifndef BRSVD_H_
#define BRSVD_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct brsvd_handle_s* brsvd_handle;

enum {
  BRSVD_OK = 0,
  BRSVD_ERR_ARG = -1,            /* null / inconsistent argument                              */
  BRSVD_ERR_BUDGET = -2,         /* device_budget_bytes (or workspace) below the working set  */
  BRSVD_ERR_ALLOC = -3,          /* hipMalloc / hipHostMalloc failed                          */
  BRSVD_ERR_HIP = -4,            /* a HIP runtime call or kernel launch failed                */
  BRSVD_ERR_ORTH_BREAKDOWN = -5, /* panel numerically rank deficient for the chosen method    */
  BRSVD_ERR_SVD_NOCONV = -6      /* Jacobi sweeps exhausted without convergence               */
};

enum { BRSVD_A_DEVICE = 0, BRSVD_A_HOST_PINNED = 1 };
enum { BRSVD_ORTH_AUTO = 0, BRSVD_ORTH_CHOLQR2 = 1, BRSVD_ORTH_TSQR = 2 };
/* How often A is read.  SEPARATE: one pass per product, 2q+2 passes, the panel re-orthonormalised
 * after every half step (the count the paper gives for a straightforward implementation, Sec. 3).
 * FUSED: while a row block is resident both products of a power step are taken from it,
 * T_I = A_I X and Z += A_I^T T_I, and the last pass forms Y_I = A_I X together with C^T += A_I^T Y_I,
 * from which B^T = C^T R^-1 (Y = Q R): q+1 passes -- the paper's "only twice" for q = 1 -- at the
 * price of one skipped re-orthonormalisation per pass (panels of condition up to (s_1/s_l)^2). */
enum { BRSVD_PASSES_SEPARATE = 0, BRSVD_PASSES_FUSED = 1 };
/* Element type of A, Omega and the results.  F32: brsvd_run and everything else.  F64 (the precision
 * the paper measures in, Sec. 4): the *_f64 entry points -- the same path on the fp64 matrix cores. */
enum { BRSVD_DTYPE_F32 = 0, BRSVD_DTYPE_F64 = 1 };

/* Problem statement of Alg. 1 / Alg. 2 (inputs A, k, p, q and the partition), plus where A
 * lives and how much device memory may be used (Sec. 4: the block size is chosen from the
 * memory available at run time). */
typedef struct {
  int64_t m, n;                 /* A is m x n                                                  */
  int32_t k, p, q;              /* target rank, oversampling, power exponent; l = k + p,
                                   1 <= l <= min(m, n, 512), k >= 1, p >= 0, q >= 0            */
  int32_t a_location;           /* BRSVD_A_DEVICE or BRSVD_A_HOST_PINNED                       */
  int64_t row_block;            /* rows per block b (last block ragged); 0 = largest block
                                   that fits the budget                                        */
  uint64_t device_budget_bytes; /* cap on all device memory owned by the handle; 0 = no cap    */
  int32_t orth_method;          /* BRSVD_ORTH_*                                                */
  int32_t pass_mode;            /* BRSVD_PASSES_*                                              */
  void* compute_stream;         /* hipStream_t for all kernels; NULL = the null stream         */
  void* copy_stream;            /* hipStream_t for host->device block copies (host-resident A);
                                   NULL = the library creates one (default priority)           */
  int32_t dtype;                /* BRSVD_DTYPE_*                                               */
  int32_t timing_level;         /* which phases brsvd_stats times (each timed phase costs two event
                                   records on the stream, about 0.1 ms per call in all):
                                   0 = every phase; 1 = pass kernels, copies and the total only,
                                   the other *_seconds fields stay 0                              */
} brsvd_params;

/* Timings are measured with HIP events recorded on compute_stream (copy_stream for the
 * copies); *_launches count kernel launches of that class during the call. */
typedef struct {
  double total_seconds;        /* whole call, first launch to last kernel completed            */
  double gemm_an_seconds;      /* Y_I = A_I * X   (sketch and power steps)                     */
  double gemm_at_seconds;      /* Z += A_I^T * Q_I (power half steps and the projection)       */
  double orth_seconds;         /* Gram, Cholesky, triangular apply (and TSQR when taken)       */
  double svd_seconds;          /* small SVD of the l x l factor                                */
  double lift_seconds;         /* U = Q*Ut, V = W*U_R, transposed store of V^T                 */
  double copy_seconds;         /* host->device block copies (sum over blocks, copy stream)     */
  double elementwise_seconds;  /* robust-PCA elementwise kernels                               */
  int64_t gemm_an_launches;
  int64_t gemm_at_launches;
  int64_t passes_over_A;       /* number of full reads of A                                    */
  int64_t bytes_A_streamed;    /* passes * element size * m * n                                */
  int32_t orth_fallbacks;      /* reruns on the TSQR route after a Cholesky breakdown (0 or 1)  */
  int32_t jacobi_sweeps;       /* sweeps of the last small SVD                                 */
  int32_t row_block;           /* rows per block actually used                                 */
  int32_t n_blocks;
} brsvd_stats;

/* Device bytes brsvd_create will allocate for these parameters (panels, partial-sum
 * scratch, small factors, and for host-resident A the two staging blocks).  Host memory. */
int brsvd_workspace_bytes(const brsvd_params* params, uint64_t* bytes_out);

/* Validates params, resolves row_block (0 => from the budget), allocates every device
 * buffer, stream and event the handle needs on the CURRENT device.  Fails with
 * BRSVD_ERR_BUDGET when device_budget_bytes is below the working set.  params is host
 * memory and is copied. */
int brsvd_create(const brsvd_params* params, brsvd_handle* handle_out);

/* One randomized SVD (Alg. 1 steps 2-6, with Omega of step 1 supplied by the caller).
 *   A      m x n fp32, leading dimension lda >= n (elements); DEVICE pointer when
 *          a_location == BRSVD_A_DEVICE, PINNED HOST pointer otherwise.  Never written.
 *   Omega  DEVICE, n x l fp32, dense (leading dimension l), i.i.d. N(0,1).  Never written.
 *   U      DEVICE out, m x l (leading dimension l): left singular vectors.
 *   S      DEVICE out, l singular values, descending, non-negative.
 *   Vt     DEVICE out, l x n (leading dimension n): right singular vectors, transposed.
 *   stats  HOST out, may be NULL.
 * Callers wanting the rank-k truncation take the first k columns / values / rows.
 * The call returns after all results are complete (it synchronises compute_stream).
 * On error the outputs are unspecified; the handle stays usable and destroyable. */
int brsvd_run(brsvd_handle h, const float* A, int64_t lda, const float* Omega,
              float* U, float* S, float* Vt, brsvd_stats* stats);

/* brsvd_run in double precision, for a handle created with dtype == BRSVD_DTYPE_F64: same arguments
 * with double elements, same pass modes, A in device or pinned host memory, same error behaviour.
 * bytes_A_streamed counts 8 bytes per element. */
int brsvd_run_f64(brsvd_handle h, const double* A, int64_t lda, const double* Omega,
                  double* U, double* S, double* Vt, brsvd_stats* stats);

/* The block-local scheme exactly as Alg. 2 prints it: the power iteration is run inside each block
 * while the block is resident, Y += (A_J A_J^T)^q A_J Omega_j (Sec. 3, Eq. (4) for the order of the
 * products), Omega_j is drawn on the device while the block is being copied (Sec. 3 "Sampling and
 * power iteration"), then Q = orth(Y), a second sweep forms B, and svd(B) is lifted.  A is read
 * twice whatever q is.  The paper cuts its input into column blocks; the row blocks of the row-major
 * A of this library are the column blocks of A^T, so the scheme is applied to A^T and the triplets
 * are swapped back: the sketch is Y (n x l) = sum_I (A_I^T A_I)^q A_I^T Omega_I with Omega m x l,
 * and B^T = A Q.  Unless q = 0 or there is one block this is a different (weaker) approximation from
 * brsvd_run's global power iteration, and without re-orthonormalisation inside a block its fp32
 * result loses the directions with (s_i / s_1)^(2q+1) below about 1e-7.
 *   seed   selects Omega = Philox4x32-10 + Box-Muller Gaussian matrix (see brsvd_philox_normal);
 *   Omega  DEVICE, m x l dense, or NULL; when given it is used instead of the generator.
 * pass_mode of the handle is ignored.  Other arguments, outputs and errors as for brsvd_run. */
int brsvd_run_alg2(brsvd_handle h, const float* A, int64_t lda, uint64_t seed, const float* Omega,
                   float* U, float* S, float* Vt, brsvd_stats* stats);

/* brsvd_run_alg2 in double precision for a handle created with dtype == BRSVD_DTYPE_F64 (Omega, when
 * drawn by the library, is then transformed in double: brsvd_philox_normal_f64). */
int brsvd_run_alg2_f64(brsvd_handle h, const double* A, int64_t lda, uint64_t seed, const double* Omega,
                       double* U, double* S, double* Vt, brsvd_stats* stats);

/* Rows [row0, row0 + rows) of the Gaussian matrix Omega(seed) with `cols` columns that
 * brsvd_run_alg2 draws, written dense to out (DEVICE, rows x cols).  Element e = row*cols + col is
 * output (e & 3) of Philox4x32-10 at counter (e >> 2) with key (seed low word, seed high word),
 * mapped to N(0,1) by Box-Muller on 23-bit uniforms ((x >> 9) + 0.5) * 2^-23: outputs 0, 1 give
 * radius*cos, radius*sin of one pair, outputs 2, 3 the second pair.  Asynchronous on `stream`. */
int brsvd_philox_normal(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, float* out,
                        void* stream);
/* The same matrix with the Box-Muller transform evaluated in double. */
int brsvd_philox_normal_f64(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, double* out,
                            void* stream);

/* Robust PCA by the inexact augmented Lagrange multiplier method, Alg. 3 / Eq. (3), with a
 * FIXED number of iterations; each iteration calls the randomized SVD above on
 * M - S_i + Y_i/mu_i, shrinks the singular values by 1/mu_i and the residual entries by
 * lambda/mu_i (shrinkage operator of Sec. 4), updates the multiplier and mu <- rho*mu.
 * The handle must have been created with a_location == BRSVD_A_DEVICE for an m x n problem.
 *   M        DEVICE, m x n fp32 dense (leading dimension n).  Never written.
 *   Omegas   DEVICE, iters x n x l fp32: one Gaussian test matrix per iteration.
 *   norm2_M  spectral norm of M (multiplier initialisation Y_0 = M / max(||M||_2,
 *            max|M_ij| / lambda)); pass <= 0 to have it estimated by one randomized SVD
 *            using Omegas[0].
 *   L, S     DEVICE out, m x n: low-rank and sparse parts.
 *   residuals HOST out (may be NULL), iters doubles: ||M-L-S||_F / ||M||_F per iteration.
 *   work     DEVICE scratch of 2*m*n floats owned by the caller (multiplier and the
 *            matrix handed to the SVD), so the handle's budget stays panel-sized.
 */
int brsvd_rpca_ialm(brsvd_handle h, const float* M, const float* Omegas, int32_t iters,
                    float lambda, float mu0, float rho, double norm2_M,
                    float* L, float* S, float* work, double* residuals, brsvd_stats* stats);

/* The same iteration with the stopping rule of Alg. 3: the loop is left after the first iteration
 * whose residual ||M-L-S||_F / ||M||_F is below tol (tol >= 0; the multiplier update of that
 * iteration is done, mu is not advanced), or after max_iters iterations.  Omegas holds max_iters
 * test matrices; residuals (HOST, may be NULL) has room for max_iters doubles, of which the first
 * *iters_done are written; iters_done (HOST, may be NULL) receives the number of iterations run.
 * brsvd_rpca_ialm is this call with tol = 0. */
int brsvd_rpca_ialm_tol(brsvd_handle h, const float* M, const float* Omegas, int32_t max_iters,
                        double tol, float lambda, float mu0, float rho, double norm2_M,
                        float* L, float* S, float* work, double* residuals, int32_t* iters_done,
                        brsvd_stats* stats);

/* The same loop in double precision (the precision of the paper's Table 2), for a handle created with
 * dtype == BRSVD_DTYPE_F64; arguments as above with double elements. */
int brsvd_rpca_ialm_tol_f64(brsvd_handle h, const double* M, const double* Omegas, int32_t max_iters,
                            double tol, double lambda, double mu0, double rho, double norm2_M,
                            double* L, double* S, double* work, double* residuals,
                            int32_t* iters_done, brsvd_stats* stats);

/* Spectral norm ||A||_2, the scale of the multiplier initialisation of Alg. 3, by the power method
 * on A^T A: x = x0/|x0|; iters times { y = A x; est = |y|; x = A^T y / |A^T y| }; *norm2_out (HOST)
 * receives the last est, a lower bound of ||A||_2 that grows with iters.  Two reads of A per
 * iteration.  A: DEVICE, m x n of the handle (a_location must be BRSVD_A_DEVICE), leading
 * dimension lda; x0: DEVICE, n floats, not zero.  Synchronises compute_stream. */
int brsvd_norm2_power(brsvd_handle h, const float* A, int64_t lda, const float* x0, int32_t iters,
                      double* norm2_out);
int brsvd_norm2_power_f64(brsvd_handle h, const double* A, int64_t lda, const double* x0, int32_t iters,
                          double* norm2_out);   /* the same for a BRSVD_DTYPE_F64 handle */

/* Frees everything the handle owns (never the caller's buffers).  NULL is allowed. */
int brsvd_destroy(brsvd_handle h);

/* Static, NUL-terminated description of a status code. */
const char* brsvd_status_string(int status);

/* ---- Individual steps of the path, exported for kernel-level parity tests and profiling.
 * All pointers are DEVICE pointers, all panels dense row-major; every call is asynchronous
 * on `stream` (a hipStream_t or NULL) except where noted.  ------------------------------ */

/* Y (rows x l) = A (rows x n, leading dimension lda) * X (n x l).  Alg. 1 step 2 / Alg. 2
 * line 4 for one row block.  scratch: DEVICE, at least brsvd_gemm_scratch_bytes(rows, n, l). */
int brsvd_gemm_an(const float* A, int64_t lda, int64_t rows, int64_t n, const float* X, int32_t l,
                  float* Y, void* scratch, uint64_t scratch_bytes, void* stream);

/* Z (n x l) (+)= A^T (A is rows x n, lda) * Q (rows x l).  Power half step Z = A^T Q and the
 * projection B^T = A^T Q (Alg. 1 step 4, Alg. 2 line 9) for one row block; accumulate != 0
 * adds to the existing Z (block-ordered accumulation). */
int brsvd_gemm_at(const float* A, int64_t lda, int64_t rows, int64_t n, const float* Q, int32_t l,
                  float* Z, int32_t accumulate, void* scratch, uint64_t scratch_bytes, void* stream);

uint64_t brsvd_gemm_scratch_bytes(int64_t rows, int64_t n, int32_t l);

/* The same two products in double precision (the precision the paper measures in, Sec. 4), on the
 * fp64 matrix cores.  Arguments as above with double elements; scratch of at least
 * brsvd_gemm_scratch_bytes_f64(rows, n, l). */
int brsvd_gemm_an_f64(const double* A, int64_t lda, int64_t rows, int64_t n, const double* X, int32_t l,
                      double* Y, void* scratch, uint64_t scratch_bytes, void* stream);
int brsvd_gemm_at_f64(const double* A, int64_t lda, int64_t rows, int64_t n, const double* Q, int32_t l,
                      double* Z, int32_t accumulate, void* scratch, uint64_t scratch_bytes, void* stream);
uint64_t brsvd_gemm_scratch_bytes_f64(int64_t rows, int64_t n, int32_t l);

/* In-place orthonormalisation of a tall panel P (rows x l, rows >= l) -- Alg. 1 step 3.
 * method is BRSVD_ORTH_*.  Optionally returns the l x l upper-triangular factor R (fp64,
 * row-major, DEVICE, may be NULL) with P_in = P_out * R.  Synchronises `stream`.
 * *fallback_taken (HOST, may be NULL) is set to 1 when AUTO switched to TSQR. */
int brsvd_orth(float* P, int64_t rows, int32_t l, int32_t method, double* R,
               int32_t* fallback_taken, void* stream);

/* One-sided Jacobi SVD of an l x l fp64 matrix R (row-major, DEVICE): R = Ur diag(S) Vr^T.
 * Outputs (DEVICE): S (l doubles, descending), Ur and Vr (l x l fp64, row-major, columns are
 * the singular vectors).  Alg. 1 step 5 applied to the triangular factor of B^T.
 * Synchronises `stream`; *sweeps (HOST, may be NULL) receives the sweep count. */
int brsvd_small_svd(const double* R, int32_t l, double* S, double* Ur, double* Vr,
                    int32_t* sweeps, void* stream);

/* brsvd_small_svd for callers that cannot allocate device memory (code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and same
 * results, but the scratch of the Jacobi iteration lives in a device array that is part of the library
 * (4 MiB per GPU the library is used on, held until the process ends), so the call makes no
 * hipMalloc / hipFree.  l <= 512 is what the array is sized for; a larger l returns BRSVD_ERR_BUDGET.
 * The address of the array is looked up on the first call on each device.  All calls on one GPU share
 * that GPU's array: calls that overlap on one GPU (different streams or threads) race and must be
 * serialised by the caller.  Nothing in the array has to be cleared between calls (every kernel writes
 * what it later reads), so a call is not affected by what an earlier, larger one left behind. */
int brsvd_small_svd_static(const double* R, int32_t l, double* S, double* Ur, double* Vr,
                           int32_t* sweeps, void* stream);

/* How the two thin products would be cut into workgroups (host-only, no GPU call): for checking the
 * plans' invariants and for reading profiles.  which = 0: Y = A X with A rows x n, out12 = {rows per
 * tile, row tiles, chunks per tile C, whole tiles, leftover tiles, main splits f, tail chunks x, tail
 * strips per workgroup j, partial panels per leftover tile, workgroups, column groups, column tiles per
 * group}.  which = 1: Z += A^T Q, out12 = {m-tiles per wave, waves, column tiles, row blocks,
 * sub-ranges per block, rows per sub-range, partial panels, chunk rows, column groups, column tiles per
 * group, 0, 0}.  out12: HOST, 12 ints. */
int brsvd_gemm_plan(int32_t which, int64_t rows, int64_t n, int32_t l, int64_t block_rows, int32_t dtype,
                    int32_t* out12);

/* Measured peaks of the device, to put next to the published ones in roofline figures (Sec. 4 of the
 * paper quotes its machine's peaks the same way).  One timed launch after one warm-up launch.
 *   kind 0: streaming read of `amount` bytes from buf (DEVICE, at least `amount` bytes);
 *   kind 1: `amount` iterations of 16 independent fp32 MFMAs (v_mfma_f32_16x16x4_f32) per wave on 2048
 *           workgroups of four waves; buf (DEVICE) receives 2048*256 floats.
 * *seconds (HOST) = duration of the launch, *work (HOST) = bytes read or flops done. */
int brsvd_probe(int32_t kind, void* buf, uint64_t amount, double* seconds, double* work, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BRSVD_H_ */
