"""Robust PCA (inexact ALM) on the GPU against the fp64 oracle and the planted decomposition."""
import numpy as np
import pytest
import torch

import paper_1706_07191_amd as B
from oracle import brsvd_oracle as O
from paper_1706_07191_amd import synth
from tests.gpu_util import need_gpu

pytestmark = pytest.mark.gpu


def _case(m, n, iters=30):
    cfg = synth.CONFIGS["C5"]
    D, L0, S0 = synth.make_rpca(cfg, m=m, n=n)
    Om = synth.rpca_omegas(cfg, n, iters)
    return cfg, D, L0, S0, Om


def test_shrink_and_update_kernels_one_iteration():
    """One ALM iteration on the GPU equals one oracle iteration (same SVD input, fp32 vs fp64)."""
    dev = need_gpu()
    cfg, D, L0, S0, Om = _case(500, 300, iters=1)
    m, n = D.shape
    lam = 1.0 / np.sqrt(max(m, n))
    n2 = float(np.linalg.norm(D.double().numpy(), 2))
    mu0 = 1.25 / n2
    h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=128))
    try:
        L, S, res, st = B.brsvd_rpca_ialm(h, D.to(dev), Om.to(dev), 1, lam, mu0, 1.5, norm2_M=n2)
    finally:
        B.brsvd_destroy(h)
    Lo, So, reso = O.rpca_ialm(D.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, 1, lam, mu0, 1.5, row_block=128)
    assert np.linalg.norm(L.double().cpu().numpy() - Lo) <= 1e-4 * np.linalg.norm(Lo)
    assert np.linalg.norm(S.double().cpu().numpy() - So) <= 1e-4 * np.linalg.norm(So)
    assert abs(res[0] - reso[0]) <= 1e-3 * reso[0]
    assert st["passes_over_A"] == 2 * cfg.q + 2 and st["elementwise_seconds"] > 0


def test_rpca_planted_recovery_matches_oracle():
    dev = need_gpu()
    cfg, D, L0, S0, Om = _case(1200, 320)
    m, n = D.shape
    lam = 1.0 / np.sqrt(max(m, n))
    n2 = float(np.linalg.norm(D.double().numpy(), 2))
    mu0 = 1.25 / n2
    h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=512))
    try:
        L, S, res, st = B.brsvd_rpca_ialm(h, D.to(dev), Om.to(dev), 30, lam, mu0, 1.5, norm2_M=n2)
        # spectral norm estimated by the library itself (one extra randomized SVD)
        L2, S2, res2, st2 = B.brsvd_rpca_ialm(h, D.to(dev), Om.to(dev), 30, lam, mu0, 1.5, norm2_M=0.0)
    finally:
        B.brsvd_destroy(h)
    Lo, So, reso = O.rpca_ialm(D.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, 30, lam, mu0, 1.5, row_block=512)
    Lg, Sg = L.double().cpu().numpy(), S.double().cpu().numpy()
    print(f"[rpca] res_gpu={res[-1]:.3e} res_oracle={reso[-1]:.3e} "
          f"L_vs_oracle={np.linalg.norm(Lg - Lo) / np.linalg.norm(Lo):.3e} "
          f"L_vs_planted={np.linalg.norm(Lg - L0.numpy()) / np.linalg.norm(L0.numpy()):.3e}", flush=True)
    assert res[-1] < 1e-5
    assert np.linalg.norm(Lg - Lo) <= 2e-3 * np.linalg.norm(Lo)
    assert np.linalg.norm(Sg - So) <= 2e-3 * np.linalg.norm(So)
    assert np.linalg.norm(Lg - L0.numpy()) <= 5e-3 * np.linalg.norm(L0.numpy())
    assert st["passes_over_A"] == 30 * (2 * cfg.q + 2)
    assert st2["passes_over_A"] == 31 * (2 * cfg.q + 2)
    assert np.linalg.norm(L2.double().cpu().numpy() - Lo) <= 5e-3 * np.linalg.norm(Lo)
    # residual history tracks the oracle's while it is above the fp32 floor
    for a, b in zip(res[:12], reso[:12]):
        assert abs(a - b) <= 2e-2 * b + 1e-6


def test_rpca_argument_errors():
    dev = need_gpu()
    cfg, D, L0, S0, Om = _case(300, 200, iters=1)
    h = B.brsvd_create(B.make_params(300, 200, cfg.k, cfg.p, cfg.q))
    try:
        with pytest.raises(B.BrsvdError):
            B.brsvd_rpca_ialm(h, D.to(dev), Om.to(dev), 1, 0.05, 1e-3, 1.0)      # rho must exceed 1
        with pytest.raises(B.BrsvdError):
            B.brsvd_rpca_ialm(h, D.to(dev), Om.to(dev), 0, 0.05, 1e-3, 1.5)      # iters >= 1
    finally:
        B.brsvd_destroy(h)


def test_config5_full_size_recovery():
    """76800 x 2000, rank-5 background + 5 % corruptions, 30 ALM iterations with k = p = 10, q = 1: the
    planted decomposition is recovered and the residual falls to the fp32 floor (properties; the fp64
    oracle of this size takes minutes and is exercised at 1200 x 320 above)."""
    dev = need_gpu()
    cfg = synth.CONFIGS["C5"]
    D, L0, S0 = synth.make_rpca(cfg, device=dev)
    Om = synth.rpca_omegas(cfg, cfg.n, 30, device=dev)
    lam = 1.0 / np.sqrt(max(cfg.m, cfg.n))
    n2 = float(torch.linalg.matrix_norm(D.double(), 2))
    h = B.brsvd_create(B.make_params(cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block))
    try:
        L, S, res, st = B.brsvd_rpca_ialm(h, D, Om, 30, lam, 1.25 / n2, 1.5, norm2_M=n2)
    finally:
        B.brsvd_destroy(h)
    assert st["passes_over_A"] == 120 and st["n_blocks"] == 10
    assert res[-1] < 1e-5 and res[-1] < res[10] < res[0]
    assert float(torch.linalg.norm(L - L0) / torch.linalg.norm(L0)) < 1e-3
    assert float(torch.linalg.norm(S - S0) / torch.linalg.norm(S0)) < 1e-3
    assert float(torch.linalg.norm(D - L - S) / torch.linalg.norm(D)) < 1e-5
