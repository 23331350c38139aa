"""brsvd_run_f64: the whole path in double precision against the fp64 oracle on the same inputs."""
import numpy as np
import pytest
import torch

import paper_1706_07191_amd as B
from oracle import brsvd_oracle as O
from paper_1706_07191_amd import synth
from tests.gpu_util import need_gpu, note

pytestmark = pytest.mark.gpu

# Both sides compute in fp64; they differ in summation order, in the orthonormaliser (CholeskyQR2 against
# Householder) and in the small SVD (one-sided Jacobi with rotation threshold 1e-13 against LAPACK), so
# agreement is limited by eps64 times the condition of the sketch panels, and the orthogonality of V =
# W_B (R V_R / sigma) by the Jacobi threshold times sigma_1 / sigma_l (a few hundred here): observed
# sigma 4e-15 .. 4e-14, U 2e-13 .. 7e-13, V 1e-12 .. 2e-11, reconstruction errors equal to 15 digits.
SIGMA_RTOL64 = 1e-11
ORTH_TOL64 = 1e-10
RECON_RTOL64 = 1e-10


def _run64(cfg, A, Om, b, **kw):
    dev = need_gpu()
    prm = B.make_params(cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, row_block=b, dtype=B.BRSVD_DTYPE_F64, **kw)
    h = B.brsvd_create(prm)
    try:
        Ad = A if not A.is_cuda and kw.get("a_location") == B.BRSVD_A_HOST_PINNED else A.to(dev)
        U, S, Vt, st = B.brsvd_run(h, Ad, Om.to(dev))
        torch.cuda.synchronize()
    finally:
        B.brsvd_destroy(h)
    return U, S, Vt, st


def _check64(A, Om, cfg, b, U, S, Vt, tag, sig_tol=SIGMA_RTOL64):
    An, On = A.numpy(), Om.numpy()
    Uo, so, Vto = O.brsvd(An, On, cfg.k, cfg.p, cfg.q, row_block=b)
    Ug, sg, Vg = U.cpu().numpy(), S.cpu().numpy(), Vt.cpu().numpy()
    k = cfg.k
    f = {"sigma_rel": float(np.max(np.abs(sg[:k] - so[:k]) / so[:k])), "orthU": O.orth_defect(Ug),
         "orthV": O.orth_defect(Vg.T), "err_gpu": O.recon_error(An, Ug, sg, Vg, k=k),
         "err_oracle": O.recon_error(An, Uo, so, Vto, k=k)}
    note(f"[f64 {tag}] " + " ".join(f"{k_}={v:.3e}" for k_, v in f.items()))
    assert U.dtype == torch.float64 and S.dtype == torch.float64
    assert np.all(np.diff(sg) <= 0) and np.all(sg >= 0)
    assert f["sigma_rel"] <= sig_tol, f
    assert f["orthU"] <= ORTH_TOL64 and f["orthV"] <= ORTH_TOL64, f
    assert abs(f["err_gpu"] - f["err_oracle"]) <= RECON_RTOL64 * f["err_oracle"], f
    return f


def _inputs(name, m, n, b):
    cfg = synth.CONFIGS[name].scaled(m, n, b)
    A = cfg.make_A().double()                      # the fp32 recipe, widened: same matrix on both sides
    A = A + 1e-9 * synth.gaussian(m, n, cfg.seed + 555, dtype=torch.float64)   # genuinely fp64 content
    Om = synth.gaussian(n, cfg.l, cfg.seed + 556, dtype=torch.float64)
    return cfg, A, Om


@pytest.mark.parametrize("name,m,n,b", [("C1", 2000, 1000, 512), ("C2", 3000, 2500, 700), ("C3", 4000, 3000, 1024),
                                         ("C4", 3000, 3500, 900), ("C1", 333, 271, 100)])
def test_f64_scaled_configs(name, m, n, b):
    cfg, A, Om = _inputs(name, m, n, b)
    U, S, Vt, st = _run64(cfg, A, Om, b)
    assert st["passes_over_A"] == 2 * cfg.q + 2 and st["orth_fallbacks"] == 0
    assert st["bytes_A_streamed"] == st["passes_over_A"] * 8 * m * n
    _check64(A, Om, cfg, b, U, S, Vt, f"{name} {m}x{n}")


def test_f64_fused_tsqr_and_streaming():
    cfg, A, Om = _inputs("C4", 2600, 1500, 640)
    U, S, Vt, st = _run64(cfg, A, Om, 640, pass_mode=B.BRSVD_PASSES_FUSED)
    assert st["passes_over_A"] == 2 * cfg.q + 2      # device-resident A: both products of a fused pass read it
    _check64(A, Om, cfg, 640, U, S, Vt, "fused", sig_tol=1e-9)
    U, S, Vt, st = _run64(cfg, A, Om, 640, orth_method=B.BRSVD_ORTH_TSQR)
    _check64(A, Om, cfg, 640, U, S, Vt, "tsqr")
    Ah = A.pin_memory()
    U, S, Vt, st = _run64(cfg, Ah, Om, 640, a_location=B.BRSVD_A_HOST_PINNED)
    assert st["copy_seconds"] > 0 and st["n_blocks"] == 5
    _check64(A, Om, cfg, 640, U, S, Vt, "host")


def test_f64_exact_rank_reaches_double_precision_error():
    """The paper reports an approximation error of 1e-15 in double precision on exactly rank-k inputs."""
    r, k, p = 12, 16, 8
    s = torch.linspace(10.0, 1.0, r, dtype=torch.float64)
    A = synth.exact_spectrum_matrix(1500, 900, s, seed=77, dtype=torch.float64)
    Om = synth.gaussian(900, k + p, 78, dtype=torch.float64)
    cfg = synth.Config("rank", 1500, 900, k, p, 1, 400, r, lambda i: i, 0.0, 0)
    U, S, Vt, st = _run64(cfg, A, Om, 400)
    sg = S.cpu().numpy()
    assert np.max(np.abs(sg[:r] - s.numpy()) / s.numpy()) < 1e-13
    err = O.recon_error(A.numpy(), U.cpu().numpy(), sg, Vt.cpu().numpy())
    note(f"[f64 exact rank] err={err:.3e} fallbacks={st['orth_fallbacks']}")
    assert err < 1e-13
    assert O.orth_defect(U.cpu().numpy()) <= 1e-10


def test_f64_dtype_mismatch_is_rejected():
    dev = need_gpu()
    cfg, A, Om = _inputs("C1", 300, 200, 100)
    h64 = B.brsvd_create(B.make_params(300, 200, cfg.k, cfg.p, cfg.q, dtype=B.BRSVD_DTYPE_F64))
    h32 = B.brsvd_create(B.make_params(300, 200, cfg.k, cfg.p, cfg.q))
    try:
        with pytest.raises(B.BrsvdError):
            B.brsvd_run(h64, A.float().to(dev), Om.float().to(dev))
        with pytest.raises(B.BrsvdError):
            B.brsvd_run(h32, A.to(dev), Om.to(dev))
        with pytest.raises(B.BrsvdError):
            B.brsvd_run_alg2(h64, A.float().to(dev), cfg.l)
        with pytest.raises(B.BrsvdError):
            B.brsvd_create(B.make_params(300, 200, cfg.k, cfg.p, cfg.q, dtype=7))
    finally:
        B.brsvd_destroy(h64)
        B.brsvd_destroy(h32)


def test_f64_seeded_random_shapes():
    """Twenty seeded random problems in double precision (shapes, block sizes, pass modes, storage)."""
    import random
    dev = need_gpu()
    rng = random.Random(64170607)
    for case in range(20):
        m = rng.choice([rng.randint(40, 400), rng.randint(400, 2500)])
        n = rng.choice([rng.randint(40, 400), rng.randint(400, 2500)])
        l = rng.randint(2, min(m, n, 140) - 1)
        p = rng.randint(0, min(l - 1, 12))
        k, q = l - p, rng.randint(0, 2)
        b = rng.choice([0, rng.randint(1, m), rng.randint(max(1, m // 8), m)])
        fused, host = rng.random() < 0.3, rng.random() < 0.25
        sig = torch.tensor([0.96 ** i for i in range(min(m, n))], dtype=torch.float64)
        A = synth.lowrank_plus_noise(m, n, sig, 1e-3, 9100 + case).double()
        A = A + 1e-9 * synth.gaussian(m, n, 9200 + case, dtype=torch.float64)
        Om = synth.gaussian(n, l, 9300 + case, dtype=torch.float64)
        cfg = synth.Config(f"rand64-{case}", m, n, k, p, q, b, min(m, n), lambda i: i, 1e-3, 9100 + case)
        kw = dict(pass_mode=B.BRSVD_PASSES_FUSED if fused else B.BRSVD_PASSES_SEPARATE)
        if host:
            kw["a_location"] = B.BRSVD_A_HOST_PINNED
        print(f"[case {case}] m={m} n={n} k={k} p={p} q={q} b={b} fused={fused} host={host}", flush=True)
        U, S, Vt, st = _run64(cfg, A.pin_memory() if host else A, Om, b, **kw)
        # the fused mode squares the condition of the sketch panels: eps64 * (sigma_1 / sigma_l)^2 is still tiny
        _check64(A, Om, cfg, b if b else m, U, S, Vt, f"rand{case}", sig_tol=1e-9 if fused else SIGMA_RTOL64)


def test_f64_rpca_matches_oracle():
    """Alg. 3 in double precision (the precision of the paper's Table 2) against the oracle: same iteration
    count under the stopping rule, L and S to 1e-7, residual history to 1e-6 relative."""
    dev = need_gpu()
    cfg = synth.CONFIGS["C5"]
    m, n = 1200, 320
    D, L0, S0 = synth.make_rpca(cfg, m=m, n=n)
    D = D.double()
    Om = synth.rpca_omegas(cfg, n, 30).double()
    lam = 1.0 / np.sqrt(max(m, n))
    n2 = float(np.linalg.norm(D.numpy(), 2))
    mu0 = 1.25 / n2
    Lo, So, reso, ito = O.rpca_ialm_tol(D.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, 30, 4e-5, lam, mu0, 1.5, row_block=512)
    h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=512, dtype=B.BRSVD_DTYPE_F64))
    try:
        L, S, res, done, st = B.brsvd_rpca_ialm_tol(h, D.to(dev), Om.to(dev), 30, 4e-5, lam, mu0, 1.5, norm2_M=n2)
        with pytest.raises(B.BrsvdError):
            B.brsvd_rpca_ialm_tol(h, D.float().to(dev), Om.float().to(dev), 30, 4e-5, lam, mu0, 1.5, norm2_M=n2)
    finally:
        B.brsvd_destroy(h)
    Lg, Sg = L.cpu().numpy(), S.cpu().numpy()
    dL, dS = np.linalg.norm(Lg - Lo) / np.linalg.norm(Lo), np.linalg.norm(Sg - So) / np.linalg.norm(So)
    note(f"[f64 rpca] iterations gpu={done} oracle={ito} L diff {dL:.3e} S diff {dS:.3e} "
         f"last residual gpu={res[-1]:.6e} oracle={reso[-1]:.6e}")
    assert L.dtype == torch.float64 and done == ito and st["passes_over_A"] == done * (2 * cfg.q + 2)
    assert dL <= 1e-7 and dS <= 1e-7
    assert np.max(np.abs(np.array(res) - reso) / reso) <= 1e-6


def test_f64_alg2_and_generator_match_oracle():
    """The block-local scheme and the device-side generator in double precision.  In fp64 even the
    configuration-2 spectrum with q = 2 ((s_1/s_k)^5 = 4e10, lost in fp32) is resolved."""
    from oracle import philox as PX
    dev = need_gpu()
    g = B.brsvd_philox_normal(2 ** 40 + 17, 257, 110, 12345, f64=True).cpu().numpy()
    o = PX.philox_normal(2 ** 40 + 17, 257, 110, 12345)
    assert np.max(np.abs(g - o) / (1.0 + np.abs(o))) <= 1e-14
    for name, m, n, b, q in (("C2", 3000, 2500, 700, 2), ("C4", 2600, 1500, 640, 1)):
        cfg = synth.CONFIGS[name].scaled(m, n, b)
        cfg.q = q
        A = cfg.make_A().double()
        seed = 2 ** 33 + 99
        Om = PX.philox_normal(seed, m, cfg.l)
        h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, q, row_block=b, dtype=B.BRSVD_DTYPE_F64))
        try:
            U, S, Vt, st = B.brsvd_run_alg2(h, A.to(dev), cfg.l, seed=seed)
        finally:
            B.brsvd_destroy(h)
        Uo, so, Vto = O.brsvd_alg2(A.numpy(), Om, cfg.k, cfg.p, q, row_block=b)
        sg, k = S.cpu().numpy(), cfg.k
        sig = float(np.max(np.abs(sg[:k] - so[:k]) / so[:k]))
        eg = O.recon_error(A.numpy(), U.cpu().numpy(), sg, Vt.cpu().numpy(), k=k)
        eo = O.recon_error(A.numpy(), Uo, so, Vto, k=k)
        note(f"[f64 alg2 {name} q={q}] sigma_rel={sig:.3e} err_gpu={eg:.6e} err_oracle={eo:.6e} "
             f"fallbacks={st['orth_fallbacks']}")
        assert st["passes_over_A"] == (2 * q + 2) * (1 + st["orth_fallbacks"])
        assert sig <= (1e-6 if q == 2 else 1e-10)         # q = 2: the sketch has condition 4e10, eps64 * that = 1e-5 at worst
        assert abs(eg - eo) <= 1e-6 * eo
        assert O.orth_defect(U.cpu().numpy()) <= ORTH_TOL64 and O.orth_defect(Vt.cpu().numpy().T) <= ORTH_TOL64


def test_f64_norm2_power_matches_oracle():
    dev = need_gpu()
    cfg = synth.CONFIGS["C5"]
    m, n = 1200, 320
    D = synth.make_rpca(cfg, m=m, n=n)[0].double()
    x0 = synth.gaussian(n, 1, cfg.seed + 99, dtype=torch.float64).reshape(-1)
    h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=256, dtype=B.BRSVD_DTYPE_F64))
    try:
        for iters in (1, 3, 20):
            got = B.brsvd_norm2_power(h, D.to(dev), x0.to(dev), iters)
            want = O.norm2_power(D.numpy(), x0.numpy(), iters)
            assert abs(got - want) <= 1e-12 * want
    finally:
        B.brsvd_destroy(h)
