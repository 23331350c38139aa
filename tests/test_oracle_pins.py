"""Pins for the CPU oracle: each test fixes the oracle to something other than itself
(a LAPACK dense SVD, a closed form, an identity, an error bound, a loop-level twin)."""
import os

import numpy as np
import pytest
import torch

from oracle import brsvd_oracle as O
from oracle import loops
from paper_1706_07191_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rel(a, b):
    return np.max(np.abs(np.asarray(a) - np.asarray(b)) / np.abs(np.asarray(b)))


def proj_equal(U, s, Vt, U2, s2, Vt2, tol):
    """Compare two factorizations through the matrices they represent (sign/rotation free)."""
    X = (U * s) @ Vt
    X2 = (U2 * s2) @ Vt2
    return np.linalg.norm(X - X2) <= tol * np.linalg.norm(X2)


def small_problem(m=60, n=40, r=12, noise=1e-3, seed=5):
    sig = torch.tensor([0.8 ** i for i in range(r)])
    A = synth.lowrank_plus_noise(m, n, sig, noise, seed).numpy()
    return A.astype(np.float64)      # exact promotion; keeps the test-side norms in fp64


# ---- P1: the Jacobi SVD and Householder QR of the loop-level twin vs LAPACK ---------------

@pytest.mark.parametrize("shape", [(5, 5), (8, 30), (20, 64), (1, 7)])
def test_jacobi_svd_matches_lapack(shape):
    rng = np.random.default_rng(3)
    B = rng.standard_normal(shape)
    U, s, Vt = loops.jacobi_svd(B)
    s_ref = np.linalg.svd(B, compute_uv=False)
    assert rel(s, s_ref) < 1e-12
    assert np.linalg.norm((U * s) @ Vt - B) < 1e-12 * np.linalg.norm(B)
    assert np.linalg.norm(U.T @ U - np.eye(shape[0])) < 1e-12
    assert np.linalg.norm(Vt @ Vt.T - np.eye(shape[0])) < 1e-12


def test_householder_qr_loops():
    rng = np.random.default_rng(4)
    Y = rng.standard_normal((50, 9))
    Q = loops.householder_qr(Y)
    assert np.linalg.norm(Q.T @ Q - np.eye(9)) < 1e-13
    # same range as Y: projecting Y onto range(Q) reproduces Y
    assert np.linalg.norm(Q @ (Q.T @ Y) - Y) < 1e-12 * np.linalg.norm(Y)


@pytest.mark.parametrize("q", [0, 1, 2])
def test_oracle_matches_loop_twin(q):
    A = small_problem()
    Om = synth.gaussian(40, 10, 11).numpy()
    U, s, Vt = O.brsvd(A, Om, 7, 3, q, row_block=16)
    U2, s2, Vt2 = loops.brsvd_loops(A, Om, 7, 3, q)
    assert rel(s, s2) < 1e-10
    assert proj_equal(U, s, Vt, U2, s2, Vt2, 1e-10)


# ---- P2: Omega = I, l = n  =>  the thin SVD of A, for any q -------------------------------

@pytest.mark.parametrize("q", [0, 1, 3])
def test_identity_sketch_is_dense_svd(q):
    rng = np.random.default_rng(7)
    A = rng.standard_normal((50, 12)) * (0.7 ** np.arange(12))
    U, s, Vt = O.brsvd(A, np.eye(12), 10, 2, q, row_block=7)
    s_ref = np.linalg.svd(A, compute_uv=False)
    assert rel(s, s_ref) < 1e-11
    assert np.linalg.norm((U * s) @ Vt - A) < 1e-12 * np.linalg.norm(A)


# ---- P3: exact recovery of a rank <= k matrix (paper: error ~1e-15 in double) ------------

@pytest.mark.parametrize("q", [0, 2])
def test_exact_recovery_rank_le_k(q):
    r, k, p = 6, 8, 4
    svals = torch.linspace(10.0, 1.0, r, dtype=torch.float64)
    A = synth.exact_spectrum_matrix(90, 70, svals, seed=21).numpy()
    Om = synth.gaussian(70, k + p, 22, dtype=torch.float64).numpy()
    U, s, Vt = O.brsvd(A, Om, k, p, q, row_block=32)
    assert rel(s[:r], svals.numpy()) < 1e-10
    assert np.all(s[r:] < 1e-10 * s[0])
    err = O.recon_error(A, U, s, Vt)
    facts = dict(line.split()[:2] for line in open(os.path.join(GOLD, "paper_facts.txt"))
                 if line.strip() and not line.startswith("#"))
    assert err < 50 * float(facts["fp64_exact_rank_error"])


# ---- P4: invariances ----------------------------------------------------------------------

def test_block_size_invariance():
    A = small_problem(m=61)
    Om = synth.gaussian(40, 10, 12).numpy()
    ref = O.brsvd(A, Om, 7, 3, 2, row_block=0)
    for b in (1, 7, 16, 61, 1000):
        out = O.brsvd(A, Om, 7, 3, 2, row_block=b)
        assert rel(out[1], ref[1]) < 1e-11
        assert proj_equal(*out, *ref, 1e-11)


def test_orth_method_invariance():
    A = small_problem()
    Om = synth.gaussian(40, 10, 13).numpy()
    ref = O.brsvd(A, Om, 7, 3, 1)
    for orth in (O.orth_cholqr2, O.orth_mgs2, loops.householder_qr):
        out = O.brsvd(A, Om, 7, 3, 1, orth=orth)
        assert rel(out[1], ref[1]) < 1e-9
        assert proj_equal(*out, *ref, 1e-9)


def test_omega_mixing_invariance():
    A = small_problem()
    Om = synth.gaussian(40, 10, 14).numpy()
    T = np.random.default_rng(1).standard_normal((10, 10)) + 3 * np.eye(10)
    ref = O.brsvd(A, Om, 7, 3, 1)
    out = O.brsvd(A, Om @ T, 7, 3, 1)
    assert rel(out[1], ref[1]) < 1e-9
    assert proj_equal(*out, *ref, 1e-9)


def test_reorth_schedule_invariance():
    """Orthonormalising once at the end (as printed in Alg. 1) or after every half step gives
    the same projection in exact arithmetic; in fp64 with q = 1 they agree to ~1e-8."""
    A = small_problem()
    Om = synth.gaussian(40, 10, 15).numpy()
    ref = O.brsvd(A, Om, 7, 3, 1, reorth=True)
    out = O.brsvd(A, Om, 7, 3, 1, reorth=False)
    assert rel(out[1][:7], ref[1][:7]) < 1e-8
    assert proj_equal(*out, *ref, 1e-7)


# ---- P5/P6/P7: identities ---------------------------------------------------------------

def test_pythagoras_interlacing_orthogonality():
    A = small_problem(m=120, n=80, r=30, noise=1e-2)
    Om = synth.gaussian(80, 20, 16).numpy()
    U, s, Vt = O.brsvd(A, Om, 15, 5, 1, row_block=50)
    # P7 orthogonality
    assert O.orth_defect(U) < 1e-12
    assert O.orth_defect(Vt.T) < 1e-12
    # P5: ||A - U S Vt||_F^2 = ||A||_F^2 - sum s_i^2 (U S Vt is an orthogonal projection of A)
    lhs = np.linalg.norm(A - (U * s) @ Vt) ** 2
    rhs = np.linalg.norm(A) ** 2 - np.sum(s ** 2)
    assert abs(lhs - rhs) < 1e-10 * np.linalg.norm(A) ** 2
    assert abs(O.recon_error(A, U, s, Vt, row_block=33) - np.sqrt(lhs) / np.linalg.norm(A)) < 1e-13
    # P6: singular values of a compression never exceed those of A
    sA = np.linalg.svd(A, compute_uv=False)
    assert np.all(s <= sA[:20] * (1 + 1e-12))
    # the triplets are consistent: A^T u_i = s_i v_i
    assert np.linalg.norm(A.T @ U - Vt.T * s) < 1e-10 * s[0]


# ---- P9: q = 0 closed form: U S Vt = P_{A Omega} A with P from a pseudo-inverse ------------

def test_q0_projector_closed_form():
    A = small_problem()
    Om = synth.gaussian(40, 10, 17).numpy()
    U, s, Vt = O.brsvd(A, Om, 7, 3, 0, row_block=9)
    Y = A @ Om
    P = Y @ np.linalg.pinv(Y)
    assert np.linalg.norm((U * s) @ Vt - P @ A) < 1e-10 * np.linalg.norm(A)


def test_q1_projector_closed_form():
    """With q = 1 the range is that of A A^T A Omega (the power-iteration formula of Sec. 2); catches a dropped or
    transposed factor in the power iteration."""
    A = small_problem()
    Om = synth.gaussian(40, 10, 18).numpy()
    U, s, Vt = O.brsvd(A, Om, 7, 3, 1, row_block=9)
    Y = A @ (A.T @ (A @ Om))
    P = Y @ np.linalg.pinv(Y)
    assert np.linalg.norm((U * s) @ Vt - P @ A) < 1e-8 * np.linalg.norm(A)


# ---- P8: Halko-Martinsson-Tropp average-case Frobenius bound (q = 0), with slack -----------

def test_hmt_bound_on_C1_shape():
    cfg = synth.CONFIGS["C1"]
    A = cfg.make_A().numpy()
    sA = np.linalg.svd(A.astype(np.float64), compute_uv=False)
    k, p = cfg.k, cfg.p
    tail = np.sqrt(np.sum(sA[k:] ** 2))
    bound = np.sqrt(1.0 + k / (p - 1.0)) * tail
    errs = []
    for t in range(3):
        Om = cfg.make_Omega(it=t).numpy()
        U, s, Vt = O.brsvd(A, Om, k, p, 0, row_block=cfg.row_block)
        e_l = O.recon_error(A, U, s, Vt) * np.linalg.norm(A.astype(np.float64))
        errs.append(e_l)
        assert e_l >= np.sqrt(np.sum(sA[k + p:] ** 2)) * (1 - 1e-9)     # Eckart-Young floor
        assert e_l <= 2.0 * bound
    assert np.mean(errs) <= 1.2 * bound
    # power iterations only tighten the error, and the rank-k truncation is close to sigma_{k+1}
    U, s, Vt = O.brsvd(A, cfg.make_Omega().numpy(), k, p, cfg.q, row_block=cfg.row_block)
    e_q = O.recon_error(A, U, s, Vt) * np.linalg.norm(A.astype(np.float64))
    assert e_q <= errs[0] * (1 + 1e-9)
    assert rel(s[:k], sA[:k]) < 1e-2


def test_hmt_spectral_bound_on_C1_shape():
    """Spectral-norm companion of the bound above (Halko, Martinsson and Tropp, the analysis the paper builds on,
    q = 0): E||A - Q Q^T A||_2 <= (1 + sqrt(k/(p-1))) sigma_{k+1} + (e sqrt(k+p)/p) (sum_{j>k} sigma_j^2)^(1/2), and its
    simplified form [1 + 4 sqrt(k+p)/(p-1) sqrt(min(m,n))] sigma_{k+1}.  A - U S V^T with all l triplets is
    A - Q Q^T A.  Slack 2 per draw (one Omega is a sample, not the expectation); the mean of three draws with 1.2."""
    cfg = synth.CONFIGS["C1"]
    A = cfg.make_A().numpy().astype(np.float64)
    sA = np.linalg.svd(A, compute_uv=False)
    k, p = cfg.k, cfg.p
    tail = np.sqrt(np.sum(sA[k:] ** 2))
    sharp = (1.0 + np.sqrt(k / (p - 1.0))) * sA[k] + np.e * np.sqrt(k + p) / p * tail
    simple = (1.0 + 4.0 * np.sqrt(k + p) / (p - 1.0) * np.sqrt(min(A.shape))) * sA[k]
    errs = []
    for t in range(3):
        Om = cfg.make_Omega(it=t).numpy()
        U, s, Vt = O.brsvd(A, Om, k, p, 0, row_block=cfg.row_block)
        e2 = np.linalg.norm(A - (U * s) @ Vt, 2)
        errs.append(e2)
        assert e2 >= sA[k + p] * (1 - 1e-9)                  # no rank-l approximation beats sigma_{l+1}
        assert e2 <= 2.0 * sharp and e2 <= 2.0 * simple
    assert np.mean(errs) <= 1.2 * sharp
    # with the configuration's power iterations the spectral error comes down towards sigma_{l+1}
    U, s, Vt = O.brsvd(A, cfg.make_Omega().numpy(), k, p, cfg.q, row_block=cfg.row_block)
    assert np.linalg.norm(A - (U * s) @ Vt, 2) <= errs[0] * (1 + 1e-9)


# ---- shrinkage operator, closed form from the paper's definition ---------------------------

def test_shrink_golden():
    rows = np.loadtxt(os.path.join(GOLD, "shrink_cases.txt"))
    for x, eps, want in rows:
        assert abs(float(O.shrink(np.array([x]), eps)[0]) - want) < 1e-15
    x = np.linspace(-3, 3, 101)
    assert np.allclose(O.shrink(x, 0.7), np.sign(x) * np.maximum(np.abs(x) - 0.7, 0.0), atol=1e-15)


# ---- argument checking ---------------------------------------------------------------------

def test_oracle_argument_errors():
    A = np.zeros((5, 4))
    with pytest.raises(ValueError):
        O.brsvd(A, np.zeros((4, 5)), 3, 2, 0)       # l > min(m, n)
    with pytest.raises(ValueError):
        O.brsvd(A, np.zeros((3, 2)), 1, 1, 0)       # Omega shape
    assert O.row_blocks(10, 4) == [(0, 4), (4, 8), (8, 10)]
    assert O.row_blocks(10, 0) == [(0, 10)]
