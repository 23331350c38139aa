"""brsvd_small_svd_static (the entry point that allocates no device memory) against brsvd_small_svd,
through the C ABI: two calls in a row on one GPU, the second with a smaller input, so that what the first
call left in the shared static scratch cannot leak into the second."""
import numpy as np
import pytest
import torch

import paper_1706_07191_amd as B
from tests.gpu_util import need_gpu

pytestmark = pytest.mark.gpu


def _matrix(l, seed, dev):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    u, _ = torch.linalg.qr(torch.randn(l, l, generator=g, dtype=torch.float64))
    v, _ = torch.linalg.qr(torch.randn(l, l, generator=g, dtype=torch.float64))
    s = torch.logspace(0, -4, l, dtype=torch.float64)
    return ((u * s) @ v.T).to(dev)


def test_small_svd_static_matches_allocating_entry_point():
    dev = need_gpu()
    # 200: block Jacobi (rows in the scratch, host-driven sweeps); 60: LDS-resident Jacobi; 1: nothing to rotate
    for l, seed in ((200, 11), (60, 12), (1, 13)):
        R = _matrix(l, seed, dev)
        print(f"[case] l={l} seed={seed}", flush=True)
        S0, Ur0, Vr0, sw0 = B.brsvd_small_svd(R)
        out = tuple(torch.full_like(t, float("nan")) for t in (S0, Ur0, Vr0))
        torch.cuda.synchronize()
        S1, Ur1, Vr1, sw1 = B.brsvd_small_svd_static(R, out=out)
        torch.cuda.synchronize()
        assert sw1 == sw0
        # same kernels on a different scratch address: the results are the same numbers
        assert torch.equal(S1, S0) and torch.equal(Ur1, Ur0) and torch.equal(Vr1, Vr0)
        # and they are an SVD of R (fp64 bar of the step: sigma 1e-9 relative against LAPACK)
        ref = np.linalg.svd(R.cpu().numpy(), compute_uv=False)
        assert np.max(np.abs(S1.cpu().numpy() - ref) / ref) <= 1e-9
        rec = (Ur1 * S1) @ Vr1.T
        assert float((rec - R).abs().max()) <= 1e-12


def test_small_svd_static_rejects_sizes_beyond_its_scratch():
    dev = need_gpu()
    l = 513
    R = torch.eye(l, dtype=torch.float64, device=dev)
    S = torch.empty(l, dtype=torch.float64, device=dev)
    Ur = torch.empty(l, l, dtype=torch.float64, device=dev)
    status = B.lib().brsvd_small_svd_static(R.data_ptr(), l, S.data_ptr(), Ur.data_ptr(), Ur.data_ptr(), None, None)
    assert status == B.BRSVD_ERR_BUDGET
    assert B.lib().brsvd_small_svd_static(None, 4, S.data_ptr(), Ur.data_ptr(), Ur.data_ptr(), None, None) == B.BRSVD_ERR_ARG
