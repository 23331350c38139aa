"""Pins for the oracle of the block-local scheme (Alg. 2 as printed) and of the counter-based
Gaussian generator both sides implement."""
import numpy as np

from oracle import brsvd_oracle as O
from oracle import philox as PX


def _lowrank(m, n, r, decay, seed, noise=0.0):
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal((m, r)) * decay ** np.arange(r)) @ rng.standard_normal((r, n))
    return A + noise * rng.standard_normal((m, n))


def _proj(U):
    return U @ U.T


# ---- Philox4x32-10 + Box-Muller ----------------------------------------------------------------

def test_philox_known_answers():
    """Known-answer vectors of Philox4x32-10 distributed with the reference implementation of
    Salmon et al. (SC'11): zero counter and key, all-ones, and the digits-of-pi vector."""
    kat = [
        ([0, 0, 0, 0], (0, 0), [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]),
        ([0xffffffff] * 4, (0xffffffff, 0xffffffff), [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]),
        ([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], (0xa4093822, 0x299f31d0),
         [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]),
    ]
    for ctr, key, want in kat:
        got = PX.philox4x32_10(np.array(ctr), key)
        assert [int(v) for v in got] == want


def test_philox_normal_is_standard_gaussian_and_windowed():
    z = PX.philox_normal(20170607, 4000, 50)
    x = z.reshape(-1)
    n = x.size
    assert abs(x.mean()) < 4 / np.sqrt(n)
    assert abs(x.var() - 1.0) < 4 * np.sqrt(2.0 / n)
    assert abs(np.mean(x ** 3)) < 4 * np.sqrt(15.0 / n)
    assert abs(np.mean(x ** 4) - 3.0) < 4 * np.sqrt(96.0 / n)
    # Kolmogorov-Smirnov distance to the normal cdf
    from math import erf
    xs = np.sort(x)
    cdf = 0.5 * (1.0 + np.vectorize(erf)(xs / np.sqrt(2.0)))
    ks = np.max(np.abs(cdf - (np.arange(n) + 0.5) / n))
    assert ks < 2.0 / np.sqrt(n)
    # columns nearly uncorrelated; the two members of a Box-Muller pair too
    C = np.corrcoef(z[:, :8], rowvar=False)
    assert np.max(np.abs(C - np.eye(8))) < 5 / np.sqrt(4000)
    # a window of rows is the same as the slice of the whole matrix; other seeds differ
    np.testing.assert_array_equal(PX.philox_normal(20170607, 37, 50, row0=1234), z[1234:1271])
    assert not np.allclose(PX.philox_normal(20170608, 10, 50), z[:10])
    # seeds beyond 32 bits reach the second key word
    assert not np.allclose(PX.philox_normal(20170607 + (1 << 32), 10, 50), z[:10])


# ---- block-local scheme ------------------------------------------------------------------------

def test_alg2_first_sweep_matches_explicit_powers():
    """Y of the first sweep against the formula with the n x n matrices (A_I^T A_I)^q formed
    explicitly (the product the right-to-left evaluation avoids)."""
    m, n, k, p, q, b = 90, 40, 6, 4, 2, 32
    A = _lowrank(m, n, 12, 0.8, 1, noise=1e-2)
    Om = np.random.default_rng(2).standard_normal((m, k + p))
    Y = np.zeros((n, k + p))
    for r0 in range(0, m, b):
        AI = A[r0:r0 + b]
        Y += np.linalg.matrix_power(AI.T @ AI, q) @ AI.T @ Om[r0:r0 + b]
    U, s, Vt = O.brsvd_alg2(A, Om, k, p, q, row_block=b)
    # range(V) = range(Y): the projector onto the computed right singular space is the one onto Y
    Qy, _ = np.linalg.qr(Y)
    assert np.linalg.norm(_proj(Vt.T) - _proj(Qy), 2) < 1e-9
    # and (U, s, Vt) is the SVD of the projection A Qy Qy^T
    Ud, sd, _ = np.linalg.svd(A @ _proj(Qy), full_matrices=False)
    np.testing.assert_allclose(s, sd[:k + p], rtol=1e-10)
    assert np.linalg.norm(U @ np.diag(s) @ Vt - A @ _proj(Qy)) < 1e-9 * np.linalg.norm(A)


def test_alg2_reduces_to_alg1_on_the_transpose():
    """q = 0 (any blocking) and a single block (any q): the block-local scheme is Alg. 1 applied to
    A^T with the same Omega, triplets swapped."""
    m, n, k, p = 120, 70, 8, 4
    A = _lowrank(m, n, 20, 0.85, 3, noise=1e-3)
    Om = np.random.default_rng(4).standard_normal((m, k + p))
    for q, b in ((0, 25), (0, 0), (1, 0), (2, 0)):
        U, s, Vt = O.brsvd_alg2(A, Om, k, p, q, row_block=b)
        U1, s1, Vt1 = O.brsvd(A.T, Om, k, p, q, row_block=17, reorth=False)
        np.testing.assert_allclose(s, s1, rtol=1e-8)
        assert np.linalg.norm(_proj(U[:, :k]) - _proj(Vt1.T[:, :k]), 2) < 1e-6
        assert np.linalg.norm(_proj(Vt.T[:, :k]) - _proj(U1[:, :k]), 2) < 1e-6


def test_alg2_equals_global_scheme_when_blocks_have_orthogonal_row_spaces():
    """If A_I A_J^T = 0 for I != J then (A^T A)^q = sum_I (A_I^T A_I)^q, so the block-local power
    iteration is the global one."""
    rng = np.random.default_rng(5)
    n, b, nb, k, p, q = 60, 30, 3, 6, 3, 2
    W, _ = np.linalg.qr(rng.standard_normal((n, n)))
    blocks = []
    for i in range(nb):                      # block i lives in its own 20-dimensional row space
        Wi = W[:, 20 * i:20 * i + 20]
        blocks.append((rng.standard_normal((b, 20)) * 0.7 ** np.arange(20)) @ Wi.T)
    A = np.vstack(blocks)
    Om = rng.standard_normal((nb * b, k + p))
    U, s, Vt = O.brsvd_alg2(A, Om, k, p, q, row_block=b)
    U1, s1, Vt1 = O.brsvd(A.T, Om, k, p, q, reorth=False)
    np.testing.assert_allclose(s, s1, rtol=1e-8)
    # with a different blocking the row spaces overlap inside a block and the results differ
    _, s2, _ = O.brsvd_alg2(A, Om, k, p, q, row_block=45)
    assert np.max(np.abs(s2 - s1) / s1) > 1e-6


def test_alg2_exact_recovery_and_basic_properties():
    m, n, k, p = 150, 90, 10, 5
    A = _lowrank(m, n, k, 0.9, 6)            # rank exactly k
    Om = np.random.default_rng(7).standard_normal((m, k + p))
    for q in (0, 1, 2):
        U, s, Vt = O.brsvd_alg2(A, Om, k, p, q, row_block=40)
        assert O.recon_error(A, U, s, Vt, k=k) < 1e-10
        assert O.orth_defect(U[:, :k]) < 1e-10 and O.orth_defect(Vt.T) < 1e-10
        assert np.all(np.diff(s) <= 1e-12) and np.all(s >= 0)
    # general input: interlacing with the true singular values, and A^T U = V S
    A = _lowrank(m, n, 40, 0.9, 8, noise=1e-3)
    sv = np.linalg.svd(A, compute_uv=False)
    U, s, Vt = O.brsvd_alg2(A, Om, k, p, 1, row_block=40)
    assert np.all(s <= sv[:k + p] * (1 + 1e-12))
    assert np.linalg.norm(A @ Vt.T - U * s) < 1e-9 * sv[0]


def test_alg2_is_a_weaker_approximation_than_the_global_power_iteration():
    """What the block-local power iteration costs: on a slowly decaying spectrum split over several
    blocks its rank-k error sits between the optimum and the q = 0 sketch, and above the global
    scheme's (which sees the whole of A A^T)."""
    m, n, k, p, q = 400, 200, 10, 5, 2
    rng = np.random.default_rng(9)
    Ul, _ = np.linalg.qr(rng.standard_normal((m, 60)))
    Vr, _ = np.linalg.qr(rng.standard_normal((n, 60)))
    A = (Ul * (1.0 / np.arange(1, 61) ** 0.5)) @ Vr.T
    errs = {"alg2": [], "alg1": [], "q0": []}
    for t in range(5):
        Om_m = np.random.default_rng(100 + t).standard_normal((m, k + p))
        U, s, Vt = O.brsvd_alg2(A, Om_m, k, p, q, row_block=50)
        errs["alg2"].append(O.recon_error(A, U, s, Vt, k=k))
        U, s, Vt = O.brsvd_alg2(A, Om_m, k, p, 0, row_block=50)
        errs["q0"].append(O.recon_error(A, U, s, Vt, k=k))
        V1, s1, U1t = O.brsvd(A.T, Om_m, k, p, q)
        errs["alg1"].append(O.recon_error(A, U1t.T, s1, V1.T, k=k))
    sv = np.linalg.svd(A, compute_uv=False)
    best = np.sqrt(np.sum(sv[k:] ** 2) / np.sum(sv ** 2))
    a2, a1, q0 = (np.mean(errs[x]) for x in ("alg2", "alg1", "q0"))
    assert best <= a1 < a2 < q0
