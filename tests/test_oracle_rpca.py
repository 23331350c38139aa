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


def test_rpca_supplied_norm2_is_the_same_iteration():
    """norm2 handed in (as the full-size GPU test does) instead of computed inside: identical results for the exact
    value; a 1 % error of it only rescales the multiplier's start and leaves the decomposition within 1e-3."""
    cfg, D, L0, S0, Om = _problem(300, 120)
    lam = 1.0 / np.sqrt(300)
    n2 = float(np.linalg.norm(D, 2))
    a = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 12, lam, 1.25 / n2, 1.5, row_block=128)
    b = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 12, lam, 1.25 / n2, 1.5, row_block=128, norm2=n2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    c = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 12, lam, 1.25 / n2, 1.5, row_block=128, norm2=1.01 * n2)
    assert np.linalg.norm(c[0] - a[0]) <= 1e-3 * np.linalg.norm(a[0])


def test_rpca_tol_stopping_rule():
    """Alg. 3's break: the loop stops at the FIRST iteration whose residual is below tol; with a
    tolerance that is never met it is the fixed-iteration loop (different code, same iterates)."""
    cfg, D, L0, S0, Om = _problem(m=300, n=120)
    m, n = D.shape
    lam = 1.0 / np.sqrt(max(m, n))
    mu0 = 1.25 / np.linalg.norm(D, 2)
    Lf, Sf, resf = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, 30, lam, mu0, 1.5)
    L0_, S0_, res0, it0 = O.rpca_ialm_tol(D, Om, cfg.k, cfg.p, cfg.q, 30, 0.0, lam, mu0, 1.5)
    assert it0 == 30
    np.testing.assert_array_equal(res0, resf)
    np.testing.assert_array_equal(L0_, Lf)
    np.testing.assert_array_equal(S0_, Sf)
    for tol in (1e-2, 1e-3, 1e-5):
        L, S, res, it = O.rpca_ialm_tol(D, Om, cfg.k, cfg.p, cfg.q, 30, tol, lam, mu0, 1.5)
        below = np.nonzero(resf < tol)[0]
        assert below.size and below[0] + 1 < 30      # the tolerance is met before the cap
        assert it == below[0] + 1 and len(res) == it # first iteration of the fixed run below tol
        np.testing.assert_array_equal(res, resf[:it])
        assert res[-1] < tol and np.all(res[:-1] >= tol)
        # the state returned is the one that passed the test: M = L + S to within tol
        assert np.linalg.norm(D - L - S) / np.linalg.norm(D) < tol
        # and it is the state of the fixed run truncated at the same iteration
        Lt, St, _ = O.rpca_ialm(D, Om, cfg.k, cfg.p, cfg.q, it, lam, mu0, 1.5)
        np.testing.assert_array_equal(L, Lt)
        np.testing.assert_array_equal(S, St)


def test_norm2_power_closed_forms():
    """Power method on A^T A.  Rank one: exact after one step.  Diagonal A = diag(d) started from
    the vector of ones: est_j = sqrt(sum d^(4j+2) / sum d^(4j)) at step j = 0, 1, ... (x_j is
    proportional to d^(2j)).  General matrix: converges to LAPACK's 2-norm from below, monotonically."""
    rng = np.random.default_rng(7)
    u = rng.standard_normal(40); v = rng.standard_normal(25)
    A1 = np.outer(u, v)
    x0 = rng.standard_normal(25)
    assert abs(O.norm2_power(A1, x0, 1) - abs(v @ x0) / np.linalg.norm(x0) * np.linalg.norm(u)) < 1e-12
    assert abs(O.norm2_power(A1, x0, 2) - np.linalg.norm(u) * np.linalg.norm(v)) < 1e-12
    d = np.array([3.0, 2.0, 1.5, 0.5, 0.1])
    for j in range(1, 6):
        est = O.norm2_power(np.diag(d), np.ones(5), j)
        closed = np.sqrt(np.sum(d ** (4 * (j - 1) + 2)) / np.sum(d ** (4 * (j - 1))))
        assert abs(est - closed) < 1e-13
    # rectangular A = [diag(d); 0] (transposed operand must not be confused with A itself)
    Ar = np.vstack([np.diag(d), np.zeros((3, 5))])
    assert abs(O.norm2_power(Ar, np.ones(5), 3) - np.sqrt(np.sum(d ** 10) / np.sum(d ** 8))) < 1e-13
    G = rng.standard_normal((200, 60)) @ np.diag(0.8 ** np.arange(60)) @ rng.standard_normal((60, 60))
    ests = [O.norm2_power(G, np.ones(60), j) for j in (1, 2, 4, 8, 16, 64)]
    assert np.all(np.diff(ests) >= -1e-12)
    assert ests[-1] <= np.linalg.norm(G, 2) * (1 + 1e-12)
    assert abs(ests[-1] - np.linalg.norm(G, 2)) / np.linalg.norm(G, 2) < 1e-6
