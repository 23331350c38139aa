"""Helpers for the GPU parity tests (not collected by pytest)."""
import os

import numpy as np
import torch

from oracle import brsvd_oracle as O

EPS32 = float(np.finfo(np.float32).eps)

# Tolerances of the GPU path against the fp64 oracle on the same fp32 inputs.
SIGMA_RTOL = 1e-4        # top-k singular values, relative
ORTH_TOL = 1e-5          # ||U^T U - I||_2
RECON_RTOL = 1e-2        # reconstruction error within 1 % of the oracle's
RECON_FLOOR = 1e-6       # ... once it is above the fp32 rounding level of the reconstruction itself (the paper
                         # reports 1e-7 for single precision on exactly representable inputs): an fp64 oracle
                         # error of 1e-15 cannot be matched to 1 % by fp32 factors


def need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a visible MI355X"
    return torch.device("cuda:0")


def note(line: str):
    """Prints a measurement line and appends it to parity.log in the run's output folder, if there is one."""
    print(line, flush=True)
    log_dir = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(log_dir):
        with open(os.path.join(log_dir, "parity.log"), "a") as f:
            f.write(line + "\n")


def check_against_oracle(A_host, Om_host, k, p, q, b, U, S, Vt, tag=""):
    """A_host / Om_host: numpy fp32; U, S, Vt: torch CUDA results.  Returns a dict of figures."""
    Uo, so, Vto = O.brsvd(A_host, Om_host, k, p, q, row_block=b)
    Ug = U.double().cpu().numpy()
    sg = S.double().cpu().numpy()
    Vg = Vt.double().cpu().numpy()
    out = {}
    out["sigma_rel"] = float(np.max(np.abs(sg[:k] - so[:k]) / so[:k]))
    out["orthU"] = O.orth_defect(Ug)
    out["orthV"] = O.orth_defect(Vg.T)
    out["err_gpu"] = O.recon_error(A_host, Ug, sg, Vg, k=k)
    out["err_oracle"] = O.recon_error(A_host, Uo, so, Vto, k=k)
    out["err_gpu_l"] = O.recon_error(A_host, Ug, sg, Vg)
    out["err_oracle_l"] = O.recon_error(A_host, Uo, so, Vto)
    line = f"[parity {tag}] " + " ".join(f"{k_}={v:.3e}" for k_, v in out.items())
    note(line)
    assert np.all(np.diff(sg) <= 0) and np.all(sg >= 0), "sigma must be descending and non-negative"
    assert out["sigma_rel"] <= SIGMA_RTOL, out
    assert out["orthU"] <= ORTH_TOL and out["orthV"] <= ORTH_TOL, out
    assert abs(out["err_gpu"] - out["err_oracle"]) <= RECON_RTOL * out["err_oracle"] + RECON_FLOOR, out
    assert abs(out["err_gpu_l"] - out["err_oracle_l"]) <= RECON_RTOL * out["err_oracle_l"] + RECON_FLOOR, out
    return out
