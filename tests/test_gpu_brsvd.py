"""End-to-end parity of brsvd_run against the fp64 oracle on the same seeded A and Omega."""
import numpy as np
import pytest
import torch

import paper_1706_07191_amd as B
from paper_1706_07191_amd import synth
from tests.gpu_util import check_against_oracle, need_gpu

pytestmark = pytest.mark.gpu


def _run(cfg, A_dev, Om_dev, row_block=None, a_location=B.BRSVD_A_DEVICE, budget=0, orth=B.BRSVD_ORTH_AUTO):
    m, n = cfg.m, cfg.n
    prm = B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block if row_block is None else row_block,
                        a_location=a_location, device_budget_bytes=budget, orth_method=orth)
    h = B.brsvd_create(prm)
    try:
        U, S, Vt, st = B.brsvd_run(h, A_dev, Om_dev)
        torch.cuda.synchronize()
    finally:
        B.brsvd_destroy(h)
    return U, S, Vt, st


def test_config1_tiny_in_core():
    dev = need_gpu()
    cfg = synth.CONFIGS["C1"]
    A = cfg.make_A()
    Om = cfg.make_Omega()
    U, S, Vt, st = _run(cfg, A.to(dev), Om.to(dev))
    assert st["passes_over_A"] == 2 * cfg.q + 2
    assert st["bytes_A_streamed"] == st["passes_over_A"] * 4 * cfg.m * cfg.n
    assert st["n_blocks"] == 4 and st["orth_fallbacks"] == 0
    check_against_oracle(A.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, cfg.row_block, U, S, Vt, "C1")


@pytest.mark.parametrize("name,m,n,b", [("C2", 3000, 2500, 700), ("C3", 4000, 3000, 1024), ("C4", 3000, 3500, 900),
                                         ("C1", 333, 271, 100)])
def test_scaled_configs_in_core(name, m, n, b):
    """The recipes of the larger configurations at sizes the oracle finishes in seconds: several
    row blocks with a ragged tail, full sketch widths (l = 110, 272, 144, 30)."""
    dev = need_gpu()
    cfg = synth.CONFIGS[name].scaled(m, n, b)
    print(f"[case] {cfg.name} l={cfg.l} q={cfg.q} b={b}", flush=True)
    A = cfg.make_A()
    Om = cfg.make_Omega()
    U, S, Vt, st = _run(cfg, A.to(dev), Om.to(dev))
    check_against_oracle(A.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, b, U, S, Vt, cfg.name)


def test_forced_tsqr_matches_oracle():
    dev = need_gpu()
    cfg = synth.CONFIGS["C2"].scaled(3000, 2500, 700)
    A = cfg.make_A()
    Om = cfg.make_Omega()
    U, S, Vt, st = _run(cfg, A.to(dev), Om.to(dev), orth=B.BRSVD_ORTH_TSQR)
    assert st["orth_fallbacks"] == 0
    check_against_oracle(A.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, 700, U, S, Vt, "C2-tsqr")


def test_block_size_independence_and_determinism():
    dev = need_gpu()
    cfg = synth.CONFIGS["C1"]
    A = cfg.make_A().to(dev)
    Om = cfg.make_Omega().to(dev)
    ref = _run(cfg, A, Om)
    again = _run(cfg, A, Om)
    assert torch.equal(ref[1], again[1]) and torch.equal(ref[0], again[0]) and torch.equal(ref[2], again[2])
    for b in (2000, 64, 777):
        out = _run(cfg, A, Om, row_block=b)
        rel = ((out[1][:cfg.k] - ref[1][:cfg.k]).abs() / ref[1][:cfg.k]).max().item()
        assert rel < 2e-5, (b, rel)


def test_host_resident_streaming_matches_in_core():
    """A in pinned host memory, streamed through the two staging buffers (ragged last block)."""
    dev = need_gpu()
    cfg = synth.CONFIGS["C4"].scaled(3000, 3500, 900)
    A = cfg.make_A()
    Om = cfg.make_Omega()
    Ap = torch.empty(cfg.m, cfg.n, dtype=torch.float32, pin_memory=True)
    Ap.copy_(A)
    U, S, Vt, st = _run(cfg, Ap, Om.to(dev), a_location=B.BRSVD_A_HOST_PINNED)
    assert st["n_blocks"] == 4 and st["gemm_an_launches"] == 4 * (cfg.q + 1)
    check_against_oracle(A.numpy(), Om.numpy(), cfg.k, cfg.p, cfg.q, 900, U, S, Vt, "C4-host")
    # budget-driven block size: working set must respect the cap
    need = B.brsvd_workspace_bytes(B.make_params(cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, row_block=256,
                                                 a_location=B.BRSVD_A_HOST_PINNED))
    U2, S2, Vt2, st2 = _run(cfg, Ap, Om.to(dev), row_block=0, a_location=B.BRSVD_A_HOST_PINNED, budget=need + (8 << 20))
    assert 256 <= st2["row_block"] < cfg.m
    rel = ((S2[:cfg.k] - S[:cfg.k]).abs() / S[:cfg.k]).max().item()
    assert rel < 2e-5


def test_exact_rank_input_fp32_error_level():
    """Exactly rank-r input, r <= k: the paper reports ~1e-7 relative error in single precision."""
    dev = need_gpu()
    r, k, p = 12, 16, 8
    s = torch.linspace(10.0, 1.0, r, dtype=torch.float64)
    A = synth.exact_spectrum_matrix(1500, 900, s, seed=77, dtype=torch.float32)
    Om = synth.gaussian(900, k + p, 78)
    cfg = synth.Config("rank", 1500, 900, k, p, 1, 400, r, lambda i: i, 0.0, 0)
    U, S, Vt, st = _run(cfg, A.to(dev), Om.to(dev))
    assert st["orth_fallbacks"] == 1 and st["passes_over_A"] == 2 * (2 * cfg.q + 2)   # the TSQR rerun
    sg = S.double().cpu().numpy()
    assert np.max(np.abs(sg[:r] - s.numpy()) / s.numpy()) < 1e-5
    assert np.all(sg[r:] < 1e-5 * sg[0])
    from oracle import brsvd_oracle as O
    err = O.recon_error(A.numpy(), U.double().cpu().numpy(), sg, Vt.double().cpu().numpy())
    assert err < 2e-6
