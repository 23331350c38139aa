"""Loop-level twin of the oracle for tiny inputs.  TEST INFRASTRUCTURE ONLY.

The same algorithm (Alg. 1) with no LAPACK factorisation: Householder QR and a one-sided
(Hestenes) Jacobi SVD written out with explicit loops, used to pin oracle/brsvd_oracle.py
(which relies on numpy.linalg) on small matrices, and pinned itself against numpy.linalg.svd.
"""
from __future__ import annotations

import numpy as np


def householder_qr(Y: np.ndarray) -> np.ndarray:
    """Thin Q (m x l) of Y by Householder reflections applied column by column."""
    R = np.array(Y, dtype=np.float64, copy=True)
    m, l = R.shape
    vs = []
    for j in range(l):
        x = R[j:, j].copy()
        alpha = -np.copysign(np.linalg.norm(x), x[0] if x[0] != 0 else 1.0)
        v = x
        v[0] -= alpha
        nv = np.linalg.norm(v)
        if nv > 0:
            v /= nv
            R[j:, j:] -= 2.0 * np.outer(v, v @ R[j:, j:])
        vs.append(v)
    Q = np.zeros((m, l))
    Q[:l, :l] = np.eye(l)
    for j in reversed(range(l)):
        v = vs[j]
        Q[j:, :] -= 2.0 * np.outer(v, v @ Q[j:, :])
    return Q


def jacobi_svd(B: np.ndarray, tol: float = 1e-15, max_sweeps: int = 60):
    """One-sided Jacobi SVD of B (r x c, r <= c): rotates the rows of B until they are mutually
    orthogonal.  Returns U (r x r), s (r,) descending, Vt (r x c) with B = U diag(s) Vt."""
    W = np.array(B, dtype=np.float64, copy=True)     # rows get orthogonalised
    r = W.shape[0]
    J = np.eye(r)                                     # accumulated rotations: W = J^T B
    for _ in range(max_sweeps):
        off = 0.0
        for a in range(r - 1):
            for b in range(a + 1, r):
                al = W[a] @ W[a]
                be = W[b] @ W[b]
                ga = W[a] @ W[b]
                if al == 0.0 or be == 0.0:
                    continue
                off = max(off, abs(ga) / np.sqrt(al * be))
                if abs(ga) <= tol * np.sqrt(al * be):
                    continue
                zeta = (be - al) / (2.0 * ga)
                t = np.sign(zeta) / (abs(zeta) + np.sqrt(1.0 + zeta * zeta)) if zeta != 0 else 1.0
                c = 1.0 / np.sqrt(1.0 + t * t)
                s = c * t
                wa, wb = W[a].copy(), W[b].copy()
                W[a], W[b] = c * wa - s * wb, s * wa + c * wb
                ja, jb = J[:, a].copy(), J[:, b].copy()
                J[:, a], J[:, b] = c * ja - s * jb, s * ja + c * jb
        if off <= tol:
            break
    s = np.linalg.norm(W, axis=1)
    order = np.argsort(-s)
    s = s[order]
    Vt = W[order] / np.where(s > 0, s, 1.0)[:, None]
    U = J[:, order]
    return U, s, Vt


def brsvd_loops(A: np.ndarray, Omega: np.ndarray, k: int, p: int, q: int):
    """Alg. 1 with plain matrix products, Householder QR and the Jacobi SVD above."""
    A = np.asarray(A, dtype=np.float64)
    Y = A @ np.asarray(Omega, dtype=np.float64)
    Q = householder_qr(Y)
    for _ in range(q):
        W = householder_qr(A.T @ Q)
        Q = householder_qr(A @ W)
    B = Q.T @ A
    Ut, s, Vt = jacobi_svd(B)
    return Q @ Ut, s, Vt
