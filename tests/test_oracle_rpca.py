"""Pins for the robust-PCA oracle (Alg. 3): planted low-rank + sparse recovery, residual
decay, and agreement with the same iteration run on an exact dense SVD."""
import numpy as np
import torch

from oracle import brsvd_oracle as O
from paper_1706_07191_amd import synth


def _problem(m=600, n=160):
    cfg = synth.CONFIGS["C5"]
    D, L0, S0 = synth.make_rpca(cfg, m=m, n=n)
    Om = synth.rpca_omegas(cfg, n, 30).numpy()
    return cfg, D.numpy().astype(np.float64), L0.numpy().astype(np.float64), S0.numpy().astype(np.float64), Om


def _ialm_dense(M, iters, lam, mu0, rho):
    """The same multiplier iteration with a full LAPACK SVD in place of the randomized one
    (singular-value thresholding as in the inexact ALM method the paper builds on)."""
    J = max(np.linalg.norm(M, 2), np.max(np.abs(M)) / lam)
    Y = M / J
    S = np.zeros_like(M)
    mu = mu0
    for _ in range(iters):
        U, s, Vt = np.linalg.svd(M - S + Y / mu, full_matrices=False)
        L = (U * np.maximum(s - 1.0 / mu, 0.0)) @ Vt
        T = M - L + Y / mu
        S = np.sign(T) * np.maximum(np.abs(T) - lam / mu, 0.0)
        Y = Y + mu * (M - L - S)
        mu *= rho
    return L, S


def test_rpca_planted_recovery_and_residuals():
    cfg, D, L0, S0, Om = _problem()
    m, n = D.shape
    lam = 1.0 / np.sqrt(max(m, n))
    mu0 = 1.25 / np.linalg.norm(D, 2)
    L, S, res = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 30, lam, mu0, 1.5, row_block=128)
    # residual ||M-L-S||_F/||M||_F decays and ends tiny
    assert res[-1] < 1e-5
    assert np.all(np.diff(res[5:]) <= 1e-12)
    # planted background recovered (noise level 1e-3 limits the accuracy)
    assert np.linalg.norm(L - L0) / np.linalg.norm(L0) < 5e-3
    # support of the corruptions found
    big = np.abs(S0) > 1.0
    assert np.mean(np.abs(S[big]) > 0) > 0.999
    assert np.linalg.matrix_rank(L, tol=1e-3 * np.linalg.norm(L, 2)) == cfg.rank   # noise triplets sit at ~1e-4 relative


def test_rpca_matches_dense_svd_iteration():
    """rank(L) = 5 < k = 10, so thresholding the randomized triplets or the exact ones gives
    the same iterates once the spectrum beyond k is below 1/mu."""
    cfg, D, L0, S0, Om = _problem(m=300, n=120)
    m, n = D.shape
    lam = 1.0 / np.sqrt(max(m, n))
    mu0 = 1.25 / np.linalg.norm(D, 2)
    L, S, _ = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 30, lam, mu0, 1.5)
    Ld, Sd = _ialm_dense(D, 30, lam, mu0, 1.5)
    assert np.linalg.norm(L - Ld) / np.linalg.norm(Ld) < 1e-3
    assert np.linalg.norm(S - Sd) / np.linalg.norm(Sd) < 1e-3
