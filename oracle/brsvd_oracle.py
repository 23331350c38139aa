"""Plain fp64 CPU oracle of the randomized SVD with power iterations, walked in row blocks.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Written from the paper, not from the
HIP code; shares nothing with it.

What it computes (Alg. 1; the sketch y = A omega and the power-iteration formula of Sec. 2; the two-sweep
block structure of Alg. 2):
    l = k + p
    Y = A Omega                      sketch                     (Alg. 1 step 2 with q = 0; Sec. 2, y = A omega)
    Q = orth(Y)                                                 (Alg. 1 step 3)
    q times:  Z = A^T Q, W = orth(Z);  Y = A W, Q = orth(Y)     (power iteration of Sec. 2; factors applied
                                                                 right to left, Sec. 3 "Implementation details")
    B = Q^T A                                                   (Alg. 1 step 4 / Alg. 2 second sweep)
    B = Ut Sigma V^T  (dense SVD)                               (Alg. 1 step 5)
    U = Q Ut                                                    (Alg. 1 step 6)
A is only ever touched one row block at a time (the paper blocks the columns of a
column-major A; a row block of a row-major A is the same memory pattern).

Readings of the paper taken here:
  * the power iteration is the global one of Alg. 1, (A A^T)^q A Omega, not the
    block-local variant printed in Alg. 2;
  * the panel is re-orthonormalised after every half step; in exact arithmetic this leaves
    range(Y), and hence U Sigma V^T, unchanged (switchable with reorth=False for the pin);
  * Omega is an input (one n x l matrix; stacking Alg. 2's per-block draws gives the same);
  * all l = k+p triplets are returned, sigma descending; callers truncate to k.

Also here: brsvd_alg2, the block-LOCAL power iteration exactly as Alg. 2 prints it (a different
approximation, kept apart from the main path; pins in tests/test_oracle_alg2.py), the robust PCA
loop of Alg. 3 with a fixed iteration count (rpca_ialm) and with its stopping rule
(rpca_ialm_tol), and the power method for ||M||_2 (norm2_power).

Pins (tests/test_oracle_*.py): dense SVD special case (Omega = I), exact recovery of a
rank <= k matrix, block-size / orth-method / Omega-mixing invariances, Pythagoras identity,
interlacing sigma_i(B) <= sigma_i(A), projector closed form for q = 0, the
Halko-Martinsson-Tropp average error bound, and a loop-level twin (oracle/loops.py).
"""
from __future__ import annotations

import numpy as np


def row_blocks(m: int, b: int):
    """Index ranges [r0, r1) of the row blocks; the last one is ragged."""
    b = m if b <= 0 else b
    return [(r0, min(m, r0 + b)) for r0 in range(0, m, b)]


def orth_householder(Y: np.ndarray) -> np.ndarray:
    """Orthonormal basis of range(Y) by Householder thin QR (LAPACK geqrf/orgqr)."""
    Q, _ = np.linalg.qr(Y, mode="reduced")
    return Q


def orth_cholqr2(Y: np.ndarray) -> np.ndarray:
    """CholeskyQR applied twice (used only to pin invariance to the orth method)."""
    for _ in range(2):
        R = np.linalg.cholesky(Y.T @ Y).T
        Y = np.linalg.solve(R.T, Y.T).T
    return Y


def orth_mgs2(Y: np.ndarray) -> np.ndarray:
    """Modified Gram-Schmidt with one re-orthogonalisation (invariance pin only)."""
    Q = np.array(Y, dtype=np.float64, copy=True)
    for j in range(Q.shape[1]):
        for _ in range(2):
            for i in range(j):
                Q[:, j] -= (Q[:, i] @ Q[:, j]) * Q[:, i]
        Q[:, j] /= np.linalg.norm(Q[:, j])
    return Q


def a_times(A, X: np.ndarray, b: int) -> np.ndarray:
    """Y[I,:] = A[I,:] X for every row block I (A promoted to fp64 a block at a time)."""
    m = A.shape[0]
    Y = np.empty((m, X.shape[1]), dtype=np.float64)
    for r0, r1 in row_blocks(m, b):
        Y[r0:r1] = np.asarray(A[r0:r1], dtype=np.float64) @ X
    return Y


def at_times(A, Q: np.ndarray, b: int) -> np.ndarray:
    """Z = sum over row blocks I of A[I,:]^T Q[I,:], accumulated in block order."""
    m, n = A.shape
    Z = np.zeros((n, Q.shape[1]), dtype=np.float64)
    for r0, r1 in row_blocks(m, b):
        Z += np.asarray(A[r0:r1], dtype=np.float64).T @ Q[r0:r1]
    return Z


def range_finder(A, Omega, q: int, row_block: int = 0, orth=orth_householder, reorth: bool = True):
    """Stage (1): orthonormal Q (m x l) with range(Q) = range((A A^T)^q A Omega)."""
    Om = np.asarray(Omega, dtype=np.float64)
    Y = a_times(A, Om, row_block)
    for _ in range(q):
        if reorth:
            Y = orth(Y)
        Z = at_times(A, Y, row_block)
        if reorth:
            Z = orth(Z)
        Y = a_times(A, Z, row_block)
    return orth(Y)


def brsvd(A, Omega, k: int, p: int, q: int, row_block: int = 0, orth=orth_householder,
          reorth: bool = True):
    """Rank-l randomized SVD of A (m x n, any float dtype; values are promoted exactly to fp64).

    Returns U (m x l), s (l,), Vt (l x n) in fp64 with s descending and non-negative."""
    m, n = A.shape
    l = k + p
    if not (1 <= l <= min(m, n)) or k < 1 or p < 0 or q < 0:
        raise ValueError("need 1 <= k, 0 <= p, 0 <= q and k+p <= min(m, n)")
    if tuple(Omega.shape) != (n, l):
        raise ValueError("Omega must be n x (k+p)")
    Q = range_finder(A, Omega, q, row_block, orth, reorth)
    Bt = at_times(A, Q, row_block)                 # B^T = A^T Q  (n x l)
    Ut, s, Vt = np.linalg.svd(Bt.T, full_matrices=False)
    U = Q @ Ut
    return U, s, Vt


# --------------------------------------------------------------------------------------
# Metrics applied identically to the oracle's and to the HIP path's results (fp64).
# --------------------------------------------------------------------------------------

def orth_defect(U: np.ndarray) -> float:
    """Spectral norm of U^T U - I."""
    U = np.asarray(U, dtype=np.float64)
    return float(np.linalg.norm(U.T @ U - np.eye(U.shape[1]), 2))


def recon_error(A, U, s, Vt, k: int | None = None, row_block: int = 4096) -> float:
    """||A - U_k diag(s_k) V_k^T||_F / ||A||_F (the accuracy measure of Sec. 4 "Results"),
    streamed over row blocks of A in fp64."""
    U = np.asarray(U, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    Vt = np.asarray(Vt, dtype=np.float64)
    if k is not None:
        U, s, Vt = U[:, :k], s[:k], Vt[:k]
    SV = s[:, None] * Vt
    num = 0.0
    den = 0.0
    for r0, r1 in row_blocks(A.shape[0], row_block):
        blk = np.asarray(A[r0:r1], dtype=np.float64)
        den += float(np.sum(blk * blk))
        blk = blk - U[r0:r1] @ SV
        num += float(np.sum(blk * blk))
    return float(np.sqrt(num / den))


# --------------------------------------------------------------------------------------
# Robust PCA by the inexact augmented Lagrange multiplier method (Alg. 3).
# --------------------------------------------------------------------------------------

def shrink(x: np.ndarray, eps: float) -> np.ndarray:
    """Shrinkage (soft-threshold) operator of Sec. 5 (defined before Alg. 3): x-eps if x>eps, x+eps if x<-eps, else 0."""
    return np.where(x > eps, x - eps, np.where(x < -eps, x + eps, 0.0))


def rpca_ialm(M, Omegas, k: int, p: int, q: int, iters: int, lam: float, mu0: float, rho: float,
              row_block: int = 0, norm2: float | None = None):
    """Alg. 3 with a fixed number of iterations.

    norm2: the value of ||M||_2 for the multiplier initialisation when the caller already has it (the dense
    2-norm of a large M takes longer than the iterations); None = computed here by LAPACK.

    Readings: S_0 = 0 (the listing initialises "E_0"); mu_i everywhere mu appears; the
    multiplier starts at Y_0 = M / max(||M||_2, ||M||_max / lam) where ||M||_max is the largest
    absolute entry; all l triplets enter L after shrinking the singular values by 1/mu_i;
    a fresh Omega (Omegas[i]) is used in iteration i.  Returns L, S, and the per-iteration
    residuals ||M - L - S||_F / ||M||_F.
    """
    M = np.asarray(M, dtype=np.float64)
    normM = np.linalg.norm(M)
    J = max(np.linalg.norm(M, 2) if norm2 is None else float(norm2), np.max(np.abs(M)) / lam)
    Y = M / J
    S = np.zeros_like(M)
    L = np.zeros_like(M)
    mu = float(mu0)
    res = []
    for i in range(iters):
        X = M - S + Y / mu
        U, s, Vt = brsvd(X, Omegas[i], k, p, q, row_block)
        L = (U * shrink(s, 1.0 / mu)) @ Vt
        S = shrink(M - L + Y / mu, lam / mu)
        Z = M - L - S
        Y = Y + mu * Z
        res.append(float(np.linalg.norm(Z) / normM))
        mu *= rho
    return L, S, np.array(res)


def rpca_ialm_tol(M, Omegas, k: int, p: int, q: int, max_iters: int, tol: float, lam: float, mu0: float,
                  rho: float, row_block: int = 0):
    """Alg. 3 with its own stopping rule: after the multiplier update of an iteration the loop is
    left as soon as ||M - L - S||_F / ||M||_F < tol (mu is not advanced any more); max_iters bounds
    the loop (Omegas must hold at least that many test matrices).  Same readings as rpca_ialm.
    Returns L, S, the residual of every iteration run, and the number of iterations run.
    """
    M = np.asarray(M, dtype=np.float64)
    normM = np.linalg.norm(M)
    J = max(np.linalg.norm(M, 2), np.max(np.abs(M)) / lam)
    Y = M / J
    S = np.zeros_like(M)
    L = np.zeros_like(M)
    mu = float(mu0)
    res = []
    i = 0
    while i < max_iters:
        U, s, Vt = brsvd(M - S + Y / mu, Omegas[i], k, p, q, row_block)
        L = (U * shrink(s, 1.0 / mu)) @ Vt
        S = shrink(M - L + Y / mu, lam / mu)
        Z = M - L - S
        Y = Y + mu * Z
        res.append(float(np.linalg.norm(Z) / normM))
        i += 1
        if res[-1] < tol:
            break
        mu = rho * mu
    return L, S, np.array(res), i


def norm2_power(A, x0, iters: int) -> float:
    """Spectral norm ||A||_2 (needed by the multiplier initialisation of Alg. 3) by the power
    method on A^T A: x <- x0 / |x0|; repeat iters times { y = A x; est = |y|; x = A^T y / |A^T y| }.
    Returns the last est (a lower bound of ||A||_2 that increases monotonically)."""
    A = np.asarray(A, dtype=np.float64)
    x = np.asarray(x0, dtype=np.float64).reshape(-1)
    x = x / np.linalg.norm(x)
    est = 0.0
    for _ in range(iters):
        y = A @ x
        est = float(np.linalg.norm(y))
        z = A.T @ y
        x = z / np.linalg.norm(z)
    return est


# --------------------------------------------------------------------------------------
# The block-local scheme as Alg. 2 prints it (power iteration inside each block).
# --------------------------------------------------------------------------------------

def brsvd_alg2(A, Omega, k: int, p: int, q: int, row_block: int = 0):
    """Alg. 2 with its block-LOCAL power iteration, on a row-major A walked in row blocks.

    The paper blocks the columns of its input; a row block A_I (b x n) of a row-major matrix is a
    column block of the transposed input, so Alg. 2 is applied to A^T (its "m" is our n):
        Y (n x l) = sum over blocks I of (A_I^T A_I)^q A_I^T Omega_I      (first sweep; Omega_I = the
                                                                           block's rows of Omega, m x l;
                                                                           factors applied right to left, Sec. 3 "Implementation details")
        Q = orth(Y)                                                       (n x l)
        B(:, I) = Q^T A_I^T  for every block                              (second sweep; B is l x m)
        B = Ut Sigma Vp^T,  Up = Q Ut                                     (SVD of B and the lift)
    so A^T ~ Up Sigma Vp^T, i.e. A ~ Vp Sigma Up^T.  Returns (U, s, Vt) = (Vp, Sigma, Up^T) for A,
    all l = k + p triplets.  No orthonormalisation happens inside a block (none is printed).
    This is a different approximation from Alg. 1 unless q = 0 or there is a single block.
    """
    m, n = A.shape
    l = k + p
    Omega = np.asarray(Omega, dtype=np.float64)
    assert Omega.shape == (m, l)
    Y = np.zeros((n, l))
    for r0, r1 in row_blocks(m, row_block):
        AI = np.asarray(A[r0:r1], dtype=np.float64)
        P = AI.T @ Omega[r0:r1]
        for _ in range(q):
            P = AI.T @ (AI @ P)
        Y += P
    Q = orth_householder(Y)
    Bt = np.empty((m, l))
    for r0, r1 in row_blocks(m, row_block):
        Bt[r0:r1] = np.asarray(A[r0:r1], dtype=np.float64) @ Q
    Ut, s, Vpt = np.linalg.svd(Bt.T, full_matrices=False)
    Up = Q @ Ut
    return Vpt.T, s, Up.T
