"""Kernel-level parity on the GPU, through the C ABI, against the fp64 oracle steps."""
import numpy as np
import pytest
import torch

import paper_1706_07191_amd as B
from oracle import brsvd_oracle as O
from oracle import loops
from paper_1706_07191_amd import synth
from tests.gpu_util import EPS32, need_gpu

pytestmark = pytest.mark.gpu


def _bound(absA, absX, K):
    # fp32 accumulation of K products: error <= c * sqrt(K) * eps * sum |a||x| (random-walk model, c = 8)
    return 8.0 * np.sqrt(K) * EPS32 * (absA @ absX) + 1e-30


GEMM_SHAPES = [  # rows, n, l
    (1000, 1000, 30),     # C1-like, ragged rows (1000 = 7*128 + 104)
    (77, 1003, 20),       # odd row length: rows at every alignment, fewer rows than a tile
    (513, 2048, 110),     # C2 width, 7 column tiles
    (300, 1024, 272),     # C3 width, 17 column tiles
    (260, 520, 300),      # two column groups
    (64, 8, 1),           # degenerate widths
    (40, 36, 36),         # l == n
    (700, 1536, 512),     # the largest sketch width
    (9000, 2100, 64),     # more row tiles than one round of workgroups: whole tiles plus a cut leftover round
]


@pytest.mark.parametrize("rows,n,l", GEMM_SHAPES)
def test_gemm_an_matches_oracle(rows, n, l):
    dev = need_gpu()
    print(f"[case] gemm_an rows={rows} n={n} l={l}", flush=True)
    A = synth.gaussian(rows, n, 101).numpy()
    X = synth.gaussian(n, l, 102).numpy()
    Y = B.brsvd_gemm_an(torch.from_numpy(A).to(dev), torch.from_numpy(X).to(dev))
    torch.cuda.synchronize()
    ref = O.a_times(A, X.astype(np.float64), b=128)
    d = np.abs(Y.double().cpu().numpy() - ref)
    assert np.all(d <= _bound(np.abs(A).astype(np.float64), np.abs(X).astype(np.float64), n))


@pytest.mark.parametrize("rows,n,l", GEMM_SHAPES)
def test_gemm_at_matches_oracle(rows, n, l):
    dev = need_gpu()
    print(f"[case] gemm_at rows={rows} n={n} l={l}", flush=True)
    A = synth.gaussian(rows, n, 103).numpy()
    Q = synth.gaussian(rows, l, 104).numpy()
    Z = B.brsvd_gemm_at(torch.from_numpy(A).to(dev), torch.from_numpy(Q).to(dev))
    torch.cuda.synchronize()
    ref = O.at_times(A, Q.astype(np.float64), b=100)
    d = np.abs(Z.double().cpu().numpy() - ref)
    assert np.all(d <= _bound(np.abs(A.T).astype(np.float64), np.abs(Q).astype(np.float64), rows))
    # accumulate flag: Z += A^T Q
    Z2 = B.brsvd_gemm_at(torch.from_numpy(A).to(dev), torch.from_numpy(Q).to(dev), Z=Z.clone(), accumulate=True)
    torch.cuda.synchronize()
    assert np.all(np.abs(Z2.double().cpu().numpy() - 2 * ref) <=
                  2 * _bound(np.abs(A.T).astype(np.float64), np.abs(Q).astype(np.float64), rows))


@pytest.mark.parametrize("rows,n,l,off", [(600, 1001, 8, 0), (600, 1002, 16, 1), (600, 1003, 40, 2), (300, 3, 3, 1),
                                          (5000, 101, 20, 3), (900, 2383, 20, 0), (1100, 1025, 110, 1),
                                          (130, 6, 5, 0), (2000, 254, 30, 1)])
def test_gemm_rows_at_any_alignment(rows, n, l, off):
    """Rows of A that start at any element address (odd row length, base pointer `off` elements past an aligned
    one): both products against the oracle, elementwise."""
    dev = need_gpu()
    print(f"[case] gemm alignment rows={rows} n={n} l={l} off={off}", flush=True)
    A = synth.gaussian(rows, n, 111).numpy()
    X = synth.gaussian(n, l, 112).numpy()
    Q = synth.gaussian(rows, l, 113).numpy()
    flat = torch.zeros(rows * n + 8, dtype=torch.float32, device=dev)
    Ad = flat[off:off + rows * n].view(rows, n)
    Ad.copy_(torch.from_numpy(A))
    assert Ad.data_ptr() % 16 == (4 * off) % 16
    Y = B.brsvd_gemm_an(Ad, torch.from_numpy(X).to(dev))
    Z = B.brsvd_gemm_at(Ad, torch.from_numpy(Q).to(dev))
    torch.cuda.synchronize()
    dy = np.abs(Y.double().cpu().numpy() - O.a_times(A, X.astype(np.float64), b=128))
    assert np.all(dy <= _bound(np.abs(A).astype(np.float64), np.abs(X).astype(np.float64), n))
    dz = np.abs(Z.double().cpu().numpy() - O.at_times(A, Q.astype(np.float64), b=100))
    assert np.all(dz <= _bound(np.abs(A.T).astype(np.float64), np.abs(Q).astype(np.float64), rows))


def test_gemm_with_row_stride():
    """A given as a view with lda > n (a column slab of a wider matrix)."""
    dev = need_gpu()
    full = synth.gaussian(300, 1200, 105)
    A = full[:, 100:900]
    X = synth.gaussian(800, 30, 106)
    Ad = full.to(dev)[:, 100:900]
    Y = B.brsvd_gemm_an(Ad, X.to(dev))
    ref = O.a_times(A.numpy(), X.numpy().astype(np.float64), b=0)
    assert np.max(np.abs(Y.double().cpu().numpy() - ref)) < 1e-3
    Q = synth.gaussian(300, 30, 107)
    Z = B.brsvd_gemm_at(Ad, Q.to(dev))
    refz = O.at_times(A.numpy(), Q.numpy().astype(np.float64), b=0)
    assert np.max(np.abs(Z.double().cpu().numpy() - refz)) < 1e-3


@pytest.mark.parametrize("rows,l,cond", [(3000, 30, 1e2), (1000, 110, 1e4), (5000, 272, 1e3), (50, 50, 10.0),
                                          (700, 1, 1.0), (3000, 512, 1e3), (2000, 130, 1e3)])
def test_orth_cholqr2(rows, l, cond):
    dev = need_gpu()
    print(f"[case] orth rows={rows} l={l} cond={cond}", flush=True)
    s = torch.logspace(0, -np.log10(cond), l, dtype=torch.float64) if l > 1 else torch.ones(1, dtype=torch.float64)
    mix, _ = torch.linalg.qr(synth.gaussian(l, l, 32, dtype=torch.float64))     # orthogonal: cond(P) = cond
    P = (synth.exact_spectrum_matrix(rows, l, s, seed=31) @ mix).float()
    Pd = P.to(dev).contiguous()
    Qd, R, fb = B.brsvd_orth(Pd, method=B.BRSVD_ORTH_CHOLQR2, want_R=True)
    Q = Qd.double().cpu().numpy()
    R = R.cpu().numpy()
    assert not fb
    assert O.orth_defect(Q) < 5e-6
    # same range as P and P = Q R with R upper triangular
    P64 = P.double().numpy()
    assert np.linalg.norm(Q @ R - P64) <= 1e-5 * np.linalg.norm(P64)
    assert np.allclose(R, np.triu(R))
    Qo = O.orth_householder(P64)
    # range(Q) = range(P) up to the fp32 rounding of P R^-1, which scales with cond(P)
    assert np.linalg.norm(Qo @ (Qo.T @ Q) - Q, 2) < 20 * EPS32 * cond


@pytest.mark.parametrize("rows,l,cond", [(3000, 30, 1e2), (2500, 110, 1e6), (5000, 272, 1e4), (1024, 16, 10.0),
                                          (1025, 64, 1e3), (40, 40, 10.0), (2100, 512, 1e3)])
def test_orth_tsqr(rows, l, cond):
    """The Householder-tree route, forced: orthonormal, same range, P = Q R with R upper triangular."""
    dev = need_gpu()
    print(f"[case] tsqr rows={rows} l={l} cond={cond}", flush=True)
    s = torch.logspace(0, -np.log10(cond), l, dtype=torch.float64)
    mix, _ = torch.linalg.qr(synth.gaussian(l, l, 34, dtype=torch.float64))
    P = (synth.exact_spectrum_matrix(rows, l, s, seed=33) @ mix).float()
    Qd, R, fb = B.brsvd_orth(P.to(dev).contiguous(), method=B.BRSVD_ORTH_TSQR, want_R=True)
    Q = Qd.double().cpu().numpy()
    R = R.cpu().numpy()
    P64 = P.double().numpy()
    assert O.orth_defect(Q) < 5e-6
    assert np.allclose(R, np.triu(R))
    assert np.linalg.norm(Q @ R - P64) <= 1e-5 * np.linalg.norm(P64)
    Qo = O.orth_householder(P64)
    assert np.linalg.norm(Qo @ (Qo.T @ Q) - Q, 2) < 20 * EPS32 * cond
    # R agrees with LAPACK's Householder factor up to row signs
    Ro = np.linalg.qr(P64, mode="r")
    assert np.linalg.norm(np.abs(R) - np.abs(Ro)) <= 1e-4 * np.linalg.norm(Ro)


def test_orth_rank_deficient_panel():
    """A panel of numerical rank r < l (the sketch of an exactly rank-r matrix, as in the paper's own test
    inputs): the first CholeskyQR sweep clamps the vanishing pivots, the second one orthonormalises the
    damped noise columns; every route returns an orthonormal basis that contains range(P), and P = Q R."""
    dev = need_gpu()
    rows, l, r = 2000, 24, 10
    G1 = synth.gaussian(rows, r, 35, dtype=torch.float64)
    G2 = synth.gaussian(r, l, 36, dtype=torch.float64)
    P = (G1 @ G2).float()
    P64 = P.double().numpy()
    for method in (B.BRSVD_ORTH_AUTO, B.BRSVD_ORTH_CHOLQR2, B.BRSVD_ORTH_TSQR):
        Qd, Rd, fb = B.brsvd_orth(P.to(dev).contiguous(), method=method, want_R=True)
        Q = Qd.double().cpu().numpy()
        assert O.orth_defect(Q) < 5e-6, method
        assert np.linalg.norm(Q @ (Q.T @ P64) - P64) <= 1e-5 * np.linalg.norm(P64), method
        assert np.linalg.norm(Q @ Rd.cpu().numpy() - P64) <= 1e-5 * np.linalg.norm(P64), method
    # an exactly repeated column
    P2 = synth.gaussian(1500, 12, 37)
    P2[:, 7] = P2[:, 3]
    Qd, Rd, fb = B.brsvd_orth(P2.to(dev).contiguous(), method=B.BRSVD_ORTH_AUTO)
    Q = Qd.double().cpu().numpy()
    assert O.orth_defect(Q) < 5e-6
    assert np.linalg.norm(Q @ (Q.T @ P2.double().numpy()) - P2.double().numpy()) <= 1e-5 * np.linalg.norm(P2.double().numpy())
    # an all-zero panel cannot be orthonormalised by any route
    with pytest.raises(B.BrsvdError):
        B.brsvd_orth(torch.zeros(100, 8, device=dev), method=B.BRSVD_ORTH_AUTO)


@pytest.mark.parametrize("l", [1, 2, 7, 30, 111, 128, 129, 272, 300, 512])
def test_small_svd_jacobi(l):
    """R is the triangular factor of a matrix with prescribed singular values (cond 1e6, about the
    largest a factor derived from fp32 data can meaningfully have)."""
    dev = need_gpu()
    print(f"[case] small_svd l={l}", flush=True)
    rng = np.random.default_rng(40 + l)
    s_true = np.logspace(0, -6, l) if l > 1 else np.ones(1)
    U0, _ = np.linalg.qr(rng.standard_normal((l, l)))
    V0, _ = np.linalg.qr(rng.standard_normal((l, l)))
    R = np.linalg.qr((U0 * s_true) @ V0.T, mode="r")
    S, Ur, Vr, sweeps = B.brsvd_small_svd(torch.from_numpy(np.ascontiguousarray(R)).to(dev))
    S, Ur, Vr = S.cpu().numpy(), Ur.cpu().numpy(), Vr.cpu().numpy()
    assert np.max(np.abs(S - s_true) / s_true) < 1e-9
    assert np.all(np.diff(S) <= 0)
    assert np.linalg.norm((Ur * S) @ Vr.T - R) < 1e-11 * np.linalg.norm(R)
    # Ur = R Vr diag(1/s): its error is the Jacobi tolerance (1e-13) times cond(R) = 1e6
    assert np.linalg.norm(Ur.T @ Ur - np.eye(l), 2) < 5e-7
    assert np.linalg.norm(Vr.T @ Vr - np.eye(l), 2) < 1e-10
    assert 1 <= sweeps <= 20 or l == 1
    if l <= 30:   # the loop-level twin agrees too
        _, s2, _ = loops.jacobi_svd(R)
        assert np.max(np.abs(S - s2) / s2) < 1e-8            # both Jacobi codes are relatively accurate


# ---- the same two products in double precision (fp64 matrix cores) ------------------------------

EPS64 = float(np.finfo(np.float64).eps)


@pytest.mark.parametrize("rows,n,l", GEMM_SHAPES)
def test_gemm_f64_matches_oracle(rows, n, l):
    """fp64 path against the fp64 oracle: elementwise within 8 sqrt(K) eps64 (|A| |X|), both products,
    the accumulate flag, and an unaligned view (rows off the 16-byte grid)."""
    dev = need_gpu()
    A = synth.gaussian(rows, n, 201, dtype=torch.float64)
    X = synth.gaussian(n, l, 202, dtype=torch.float64)
    Q = synth.gaussian(rows, l, 203, dtype=torch.float64)
    An, Xn, Qn = A.numpy(), X.numpy(), Q.numpy()
    Y = B.brsvd_gemm_an(A.to(dev), X.to(dev))
    assert Y.dtype == torch.float64
    ref = O.a_times(An, Xn, b=128)
    assert np.all(np.abs(Y.cpu().numpy() - ref) <= 8.0 * np.sqrt(n) * EPS64 * (np.abs(An) @ np.abs(Xn)) + 1e-300)
    Z = B.brsvd_gemm_at(A.to(dev), Q.to(dev))
    refz = O.at_times(An, Qn, b=100)
    bz = 8.0 * np.sqrt(rows) * EPS64 * (np.abs(An.T) @ np.abs(Qn)) + 1e-300
    assert np.all(np.abs(Z.cpu().numpy() - refz) <= bz)
    Z2 = B.brsvd_gemm_at(A.to(dev), Q.to(dev), Z=Z.clone(), accumulate=True)
    assert np.all(np.abs(Z2.cpu().numpy() - 2 * refz) <= 2 * bz)
    if n > 8:
        Av = A.to(dev)[:, 1:n - 2]          # odd offset: rows not 32-byte aligned
        Yv = B.brsvd_gemm_an(Av, X.to(dev)[1:n - 2].contiguous())
        refv = An[:, 1:n - 2] @ Xn[1:n - 2]
        assert np.max(np.abs(Yv.cpu().numpy() - refv)) <= 1e-11 * max(1.0, np.max(np.abs(refv)))
