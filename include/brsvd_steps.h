/*
 * brsvd_steps.h -- the individual steps of the block randomized SVD path of libbrsvd, exported for
 * kernel-level parity tests, profiling and benchmarks.  brsvd.h holds the product calls.
 *
 * All pointers are DEVICE pointers unless marked HOST, all panels dense row-major; every call returns
 * an int status as in brsvd.h and is asynchronous on `stream` (a hipStream_t or NULL) except where
 * noted.  No call here allocates device memory: scratch is the caller's.
 */
#ifndef BRSVD_STEPS_H_
#define BRSVD_STEPS_H_

#include "brsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Y (rows x l) = A (rows x n, leading dimension lda) * X (n x l).  Alg. 1 step 2 / Alg. 2
 * line 4 for one row block.  scratch: at least brsvd_gemm_scratch_bytes(rows, n, l). */
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
 * row-major, may be NULL) with P_in = P_out * R.  scratch: at least brsvd_orth_scratch_bytes(rows, l),
 * 256-byte aligned; too small a scratch returns BRSVD_ERR_BUDGET.  Synchronises `stream`.
 * *fallback_taken (HOST, may be NULL) is set to 1 when AUTO switched to TSQR. */
int brsvd_orth(float* P, int64_t rows, int32_t l, int32_t method, double* R,
               int32_t* fallback_taken, void* scratch, uint64_t scratch_bytes, void* stream);
uint64_t brsvd_orth_scratch_bytes(int64_t rows, int32_t l);

/* One-sided Jacobi SVD of an l x l fp64 matrix R (row-major): R = Ur diag(S) Vr^T.
 * Outputs: S (l doubles, descending), Ur and Vr (l x l fp64, row-major, columns are the singular
 * vectors).  Alg. 1 step 5 applied to the triangular factor of B^T.  scratch: at least
 * brsvd_small_svd_scratch_bytes(l), 256-byte aligned (BRSVD_ERR_BUDGET otherwise); its contents need
 * no initialisation.  Synchronises `stream`; *sweeps (HOST, may be NULL) receives the sweep count. */
int brsvd_small_svd(const double* R, int32_t l, double* S, double* Ur, double* Vr,
                    int32_t* sweeps, void* scratch, uint64_t scratch_bytes, void* stream);
uint64_t brsvd_small_svd_scratch_bytes(int32_t l);

/* brsvd_small_svd for callers that cannot allocate device memory or carry a workspace (code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same kernels and
 * same results, but the scratch of the Jacobi iteration lives in a device array that is part of the
 * library (4 MiB per GPU the library is used on, held until the process ends), so neither the caller
 * nor the call allocates anything.  l <= 512 is what the array is sized for; a larger l returns
 * BRSVD_ERR_BUDGET.  The address of the array is looked up on the first call on each device.  All
 * calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or
 * threads) race and must be serialised by the caller.  Nothing in the array has to be cleared between
 * calls (every kernel writes what it later reads), so a call is not affected by what an earlier,
 * larger one left behind. */
int brsvd_small_svd_static(const double* R, int32_t l, double* S, double* Ur, double* Vr,
                           int32_t* sweeps, void* stream);

/* How the two thin products would be cut into workgroups (host-only, no GPU call): for checking the
 * plans' invariants and for reading profiles.  which = 0: Y = A X with A rows x n, out12 = {rows per
 * tile, row tiles, chunks per tile C, whole tiles, leftover tiles, main splits f, tail chunks x, tail
 * strips per workgroup j, partial panels per leftover tile, workgroups, column groups, column tiles per
 * group}.  which = 1: Z += A^T Q, out12 = {m-tiles per wave, waves, column tiles, row blocks,
 * sub-ranges per block, rows per sub-range, partial panels, chunk rows, column groups, column tiles per
 * group, 0, 0}.  which = 2: bytes of split-sum scratch, out12 = {A X: low 31 bits, high bits, A^T Q: low
 * 31 bits, high bits, 0, ...}.  out12: HOST, 12 ints. */
int brsvd_gemm_plan(int32_t which, int64_t rows, int64_t n, int32_t l, int64_t block_rows, int32_t dtype,
                    int32_t* out12);

/* Measurement helper, not a step of the method: measured peaks of the device, to put next to the
 * published ones in roofline figures.  One timed launch after one warm-up launch; synchronous.
 *   kind 0: streaming read of `amount` bytes from buf (at least `amount` bytes);
 *   kind 1: `amount` iterations of 16 independent fp32 MFMAs (v_mfma_f32_16x16x4_f32) per wave on 2048
 *           workgroups of four waves; buf receives 2048*256 floats.
 * *seconds (HOST) = duration of the launch, *work (HOST) = bytes read or flops done. */
int brsvd_probe(int32_t kind, void* buf, uint64_t amount, double* seconds, double* work, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BRSVD_STEPS_H_ */
