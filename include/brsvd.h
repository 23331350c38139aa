/*
 * brsvd.h -- C ABI of the MI355X (gfx950) block randomized SVD library.
 *
 * The library computes the rank-l (l = k + p) randomized SVD of an m x n matrix A by the two-stage
 * scheme of Alg. 1 of the paper (sketch Y = A*Omega, q power iterations with A*A^T, orthonormal
 * basis Q, projection B = Q^T*A, small SVD of B, lift U = Q*Ut), with A visited one row block at a
 * time and only the thin panels (m x l, n x l) kept on the device, as in the block method of
 * Alg. 2 / Sec. 3.  A may live in device memory or in pinned host memory; in the latter case row
 * blocks are streamed through two staging buffers on a copy stream while the previous block is
 * being multiplied.
 *
 * All matrices are ROW-MAJOR.  All entry points return an int status (0 = success, negative =
 * error), never throw, and never abort.  The library is not re-entrant per handle: one call at a
 * time per handle.  The individual steps of the path (thin products, orthonormalisation, small
 * SVD) are exported separately in brsvd_steps.h.
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
  BRSVD_ERR_BUDGET = -2,         /* device_budget_bytes, workspace or scratch below the need  */
  BRSVD_ERR_ALLOC = -3,          /* a host or device allocation failed                        */
  BRSVD_ERR_HIP = -4,            /* a HIP runtime call or kernel launch failed                */
  BRSVD_ERR_ORTH_BREAKDOWN = -5, /* panel numerically rank deficient for the chosen method    */
  BRSVD_ERR_SVD_NOCONV = -6      /* Jacobi sweeps exhausted without convergence               */
};

enum { BRSVD_A_DEVICE = 0, BRSVD_A_HOST_PINNED = 1 };
enum { BRSVD_ORTH_AUTO = 0, BRSVD_ORTH_CHOLQR2 = 1, BRSVD_ORTH_TSQR = 2 };
/* How the products of a power step are scheduled.  SEPARATE: one pass over A per product, 2q+2
 * passes, the panel re-orthonormalised after every half step (the count the paper gives for a
 * straightforward implementation, Sec. 3).  FUSED: both products of a power step are taken from a
 * row block while it is resident in its staging buffer, T_I = A_I X and Z += A_I^T T_I, and the last
 * pass forms Y_I = A_I X together with C^T += A_I^T Y_I, from which B^T = C^T R^-1 (Y = Q R): a
 * host-resident A crosses the host link q+1 times -- the paper's "only twice" for q = 1 -- at the
 * price of one skipped re-orthonormalisation per pass (panels of condition up to (s_1/s_l)^2).  For a
 * device-resident A the two products are two kernels that each read A from device memory, so FUSED
 * saves orthonormalisations there, not reads.  The fused projection multiplies the rounding noise of
 * C^T by (s_1/s_l)^2, so it only holds the accuracy of the separate mode while s_l/s_1 stays well above
 * the square root of the machine epsilon; the library checks this on the triangular factor R of the
 * sketch and, when min |R_ii| / max |R_ii| is below 3e-4 (fp32) or 3e-8 (fp64), repeats the run with
 * separate passes (stats.fused_fallbacks). */
enum { BRSVD_PASSES_SEPARATE = 0, BRSVD_PASSES_FUSED = 1 };
/* Element type of A, Omega and the results.  F32: brsvd_run and everything else.  F64 (the precision
 * the paper measures in, Sec. 4 "Experiments"): the *_f64 entry points -- the same path on the fp64
 * matrix cores. */
enum { BRSVD_DTYPE_F32 = 0, BRSVD_DTYPE_F64 = 1 };

/* Problem statement of Alg. 1 / Alg. 2 (inputs A, k, p, q and the partition), plus where A lives and
 * how much device memory may be used (Sec. 4 "Experiment environment and setup": the block size is
 * chosen from the memory available at run time). */
typedef struct {
  int64_t m, n;                 /* A is m x n                                                  */
  int32_t k, p, q;              /* target rank, oversampling, power exponent; l = k + p,
                                   1 <= l <= min(m, n, 512), k >= 1, p >= 0, q >= 0            */
  int32_t a_location;           /* BRSVD_A_DEVICE or BRSVD_A_HOST_PINNED                       */
  int64_t row_block;            /* rows per block b (last block ragged); 0 = largest block
                                   that fits the budget                                        */
  uint64_t device_budget_bytes; /* cap on all device memory the handle uses; 0 = no cap        */
  int32_t orth_method;          /* BRSVD_ORTH_*                                                */
  int32_t pass_mode;            /* BRSVD_PASSES_*                                              */
  void* compute_stream;         /* hipStream_t for all kernels; NULL = the null stream         */
  void* copy_stream;            /* hipStream_t for host->device block copies (host-resident A);
                                   NULL = the library creates one (default priority)           */
  int32_t dtype;                /* BRSVD_DTYPE_*                                               */
  int32_t timing_level;         /* which phases brsvd_stats times (each timed phase costs two event
                                   records on the stream, about 0.1 ms per call in all):
                                   0 = every phase; 1 = pass kernels, copies, the robust-PCA update
                                   kernel and the total only, the other *_seconds fields stay 0   */
  void* workspace;              /* DEVICE, optional: memory the handle uses instead of allocating its
                                   own (panels, split-sum scratch, small factors, staging blocks).
                                   256-byte aligned, at least brsvd_workspace_bytes(); owned by the
                                   caller and not freed by brsvd_destroy.  NULL = the library
                                   allocates (one hipMalloc in brsvd_create)                      */
  uint64_t workspace_bytes;     /* size of workspace; ignored when workspace is NULL              */
} brsvd_params;

/* Timings are measured with HIP events recorded on compute_stream (copy_stream for the copies);
 * *_launches count kernel launches of that class during the call. */
typedef struct {
  double total_seconds;        /* whole call, first launch to last kernel completed            */
  double gemm_an_seconds;      /* Y_I = A_I * X   (sketch and power steps), the product kernels only */
  double gemm_at_seconds;      /* Z += A_I^T * Q_I (power half steps and the projection), likewise   */
  double orth_seconds;         /* Gram, Cholesky, triangular apply (and TSQR when taken)       */
  double svd_seconds;          /* small SVD of the l x l factor                                */
  double lift_seconds;         /* U = Q*Ut, V = W*U_R, transposed store of V^T                 */
  double copy_seconds;         /* host->device block copies (sum over blocks, copy stream)     */
  double elementwise_seconds;  /* robust-PCA elementwise kernels (norms, initialisation, update,
                                  residual sum, final low-rank product)                         */
  int64_t gemm_an_launches;
  int64_t gemm_at_launches;
  int64_t passes_over_A;       /* full reads of A from the memory it lives in: over the host link for
                                  a host-resident A, from device memory by the product kernels
                                  otherwise (bytes_A_streamed / (element size * m * n))          */
  int64_t bytes_A_streamed;    /* bytes of A read from the memory it lives in                   */
  int32_t orth_fallbacks;      /* reruns on the TSQR route after a Cholesky breakdown (0 or 1)  */
  int32_t jacobi_sweeps;       /* sweeps of the last small SVD                                 */
  int32_t row_block;           /* rows per block actually used                                 */
  int32_t n_blocks;
  double split_sum_seconds;    /* kernels that add the partial panels of split products (both products) */
  double rpca_update_seconds;  /* the fused robust-PCA update kernel alone (part of elementwise_seconds) */
  int64_t rpca_update_launches;
  int64_t bytes_A_read_by_kernels; /* bytes of A, or of its staged blocks, read from device memory by the
                                      product kernels (equals bytes_A_streamed for a device-resident A) */
  int32_t fused_fallbacks;     /* reruns with separate passes after a fused run whose sketch was too ill
                                  conditioned for the fused projection (see BRSVD_PASSES_FUSED)          */
  int32_t reserved_;
} brsvd_stats;

/* Device bytes a handle needs for these parameters (panels, partial-sum scratch, small factors, and
 * for host-resident A the two staging blocks): what brsvd_create allocates, or the least size of a
 * caller's workspace.  Host memory. */
int brsvd_workspace_bytes(const brsvd_params* params, uint64_t* bytes_out);

/* Validates params, resolves row_block (0 => from the budget), takes the device memory (params->workspace,
 * else one allocation), and creates the stream and events the handle needs on the CURRENT device.
 * Fails with BRSVD_ERR_BUDGET when device_budget_bytes or workspace_bytes is below the working set.
 * params is host memory and is copied. */
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
 * The call returns after all results are complete (it synchronises compute_stream); when it returns an
 * error, too, no work of the call is left running on either stream.
 * On error the outputs are unspecified; the handle stays usable and destroyable. */
int brsvd_run(brsvd_handle h, const float* A, int64_t lda, const float* Omega,
              float* U, float* S, float* Vt, brsvd_stats* stats);

/* brsvd_run in double precision, for a handle created with dtype == BRSVD_DTYPE_F64: same arguments
 * with double elements, same pass modes, A in device or pinned host memory, same error behaviour.
 * bytes_A_streamed counts 8 bytes per element. */
int brsvd_run_f64(brsvd_handle h, const double* A, int64_t lda, const double* Omega,
                  double* U, double* S, double* Vt, brsvd_stats* stats);

/* The block-local scheme exactly as Alg. 2 prints it: the power iteration is run inside each block
 * while the block is resident, Y += (A_J A_J^T)^q A_J Omega_j, with the factors applied from right to
 * left (Sec. 3 "Implementation details"), Omega_j is drawn on the device while the block is being
 * copied (same paragraph), then Q = orth(Y), a second sweep forms B, and svd(B) is lifted.  A host-
 * resident A crosses the host link twice whatever q is.  The paper cuts its input into column blocks;
 * the row blocks of the row-major A of this library are the column blocks of A^T, so the scheme is
 * applied to A^T and the triplets are swapped back: the sketch is Y (n x l) = sum_I (A_I^T A_I)^q
 * A_I^T Omega_I with Omega m x l, and B^T = A Q.  Unless q = 0 or there is one block this is a
 * different (weaker) approximation from brsvd_run's global power iteration, and without
 * re-orthonormalisation inside a block its fp32 result loses the directions with
 * (s_i / s_1)^(2q+1) below about 1e-7.
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
 * brsvd_run_alg2 draws (Sec. 3 "Implementation details": the test matrix is generated on the GPU),
 * written dense to out (DEVICE, rows x cols).  Element e = row*cols + col is output (e & 3) of
 * Philox4x32-10 at counter (e >> 2) with key (seed low word, seed high word), mapped to N(0,1) by
 * Box-Muller on 23-bit uniforms ((x >> 9) + 0.5) * 2^-23: outputs 0, 1 give radius*cos, radius*sin of
 * one pair, outputs 2, 3 the second pair.  Asynchronous on `stream`. */
int brsvd_philox_normal(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, float* out,
                        void* stream);
/* The same matrix with the Box-Muller transform evaluated in double. */
int brsvd_philox_normal_f64(uint64_t seed, int64_t row0, int64_t rows, int32_t cols, double* out,
                            void* stream);

/* Robust PCA by the inexact augmented Lagrange multiplier method (Alg. 3; the decomposition problem
 * and the shrinkage operator of Sec. 5), with a FIXED number of iterations; each iteration calls the
 * randomized SVD above on M - S_i + Y_i/mu_i, shrinks the singular values by 1/mu_i and the residual
 * entries by lambda/mu_i, updates the multiplier and mu <- rho*mu.
 * The handle must have been created with a_location == BRSVD_A_DEVICE for an m x n problem.
 *   M        DEVICE, m x n fp32 dense (leading dimension n).  Never written.
 *   Omegas   DEVICE, iters x n x l fp32: one Gaussian test matrix per iteration.
 *   norm2_M  spectral norm of M (multiplier initialisation Y_0 = M / max(||M||_2,
 *            max|M_ij| / lambda)); pass <= 0 to have it estimated by one randomized SVD
 *            using Omegas[0].
 *   L, S     DEVICE out, m x n: low-rank and sparse parts of the last iteration run; both are written once, after
 *            the loop (an iteration stores neither), and L serves as working storage for the multiplier while
 *            the loop runs.  L, S, work and M must not overlap.
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

/* Frees everything the handle owns (never the caller's buffers or workspace).  NULL is allowed. */
int brsvd_destroy(brsvd_handle h);

/* Static, NUL-terminated description of a status code. */
const char* brsvd_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BRSVD_H_ */
