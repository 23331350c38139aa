#!/usr/bin/env python3
"""Benchmark of the block randomized SVD hot path on one MI355X.

A "step" is one complete rank-k BRSVD (all passes over A, orthonormalisations, small SVD, lifts)
of the in-core square configuration: A fp32 20000 x 20000 (rank-200 Gaussian factors, sigma_i = 1/i,
+1e-4 noise), k = 100, p = 10, q = 2, row block 4096, with A and Omega resident in HBM before the
timed region.  Prints ONE JSON line: GB/s of A streamed per BRSVD (passes * 4*m*n bytes / seconds),
the roofline of the dominant kernel measured with HIP events inside the library, and the fp64 CPU
oracle timed on this machine's host cores as a baseline.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_MFMA_F32_TFLOPS = 157.3  # dense fp32 MFMA
PEAK_MFMA_F64_TFLOPS = 78.6   # dense fp64 MFMA
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by a plain
# 1 GiB copy (profiles/gemm_thin_C2_hbm_traffic.md).  Counters cannot be read from inside the timed run.
MEASURED_HBM_TRAFFIC = {"C2:gemm_an": 1.725e9, "C2:gemm_at": 1.850e9}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused", action="store_true",
                    help="q+1 fused passes over A instead of the 2q+2 separate ones the headline metric is quoted on")
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"],
                    help="f64 runs the same workload in double precision (brsvd_run_f64); the headline metric is f32")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (outside the timed region) so that a rocprofv3 "
                         "--pmc run has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no multi-GPU sharding or collectives); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1706_07191_amd as B
    from paper_1706_07191_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()   # fail loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    m, n, k, p, q, l = cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, cfg.l

    f64 = args.dtype == "f64"
    tdt = torch.float64 if f64 else torch.float32
    esz = 8 if f64 else 4
    A = cfg.make_A(device=dev)
    Om = cfg.make_Omega(device=dev)
    if f64:
        A = A.double()
        Om = Om.double()
    torch.cuda.synchronize()

    prm = B.make_params(m, n, k, p, q, row_block=cfg.row_block,
                        pass_mode=B.BRSVD_PASSES_FUSED if args.fused else B.BRSVD_PASSES_SEPARATE,
                        dtype=B.BRSVD_DTYPE_F64 if f64 else B.BRSVD_DTYPE_F32,
                        timing_level=1)     # the timed region times the pass kernels and the total only
    h = B.brsvd_create(prm)
    U = torch.empty(m, l, device=dev, dtype=tdt)
    S = torch.empty(l, device=dev, dtype=tdt)
    Vt = torch.empty(l, n, device=dev, dtype=tdt)
    for _ in range(args.warmup):
        B.brsvd_run(h, A, Om, U, S, Vt, want_stats=False)
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.ones(1 << 28, device=dev)          # 1 GiB of fp32
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # timed region: exactly K steps, statistics (HIP events inside the library) collected live
    acc = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        _, _, _, st = B.brsvd_run(h, A, Om, U, S, Vt, want_stats=True)
        for key, val in st.items():
            acc[key] = acc.get(key, 0) + val if key.endswith(("seconds", "launches")) else val
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = (t1 - t0) / args.steps
    passes = q + 1 if args.fused else 2 * q + 2
    bytes_a = passes * float(esz) * m * n
    gbs = bytes_a / sec / 1e9

    # dominant kernel: whichever thin GEMM took longer in total
    an_t, at_t = acc["gemm_an_seconds"], acc["gemm_at_seconds"]
    an_n, at_n = acc["gemm_an_launches"], acc["gemm_at_launches"]
    if an_t >= at_t:
        kname, kt, kn = "gemm_an", an_t, an_n
    else:
        kname, kt, kn = "gemm_at", at_t, at_n
    avg = kt / max(kn, 1)
    flops_launch = 2.0 * m * n * l            # algorithmic flops of one launch (device-resident A: all of A)
    bytes_launch = float(esz) * m * n + float(esz) * (m + n) * l
    ai = flops_launch / bytes_launch
    peak_mfma = PEAK_MFMA_F64_TFLOPS if f64 else PEAK_MFMA_F32_TFLOPS
    ridge = peak_mfma * 1e12 / (PEAK_HBM_GBS * 1e9)
    traffic = None if f64 else MEASURED_HBM_TRAFFIC.get(f"{args.config}:{kname}")
    if ai >= ridge:
        ach = flops_launch / avg / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": peak_mfma, "unit": "TFLOP/s",
                "frac": ach / peak_mfma, "traffic": traffic}
    else:
        ach = bytes_launch / avg / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": traffic}
    roof.update({"kernel": kname, "avg_launch_ms": avg * 1e3, "launches_per_step": kn / args.steps,
                 "hbm_GBps": bytes_launch / avg / 1e9, "hbm_frac": bytes_launch / avg / 1e9 / PEAK_HBM_GBS,
                 "mfma_TFLOPs": flops_launch / avg / 1e12,
                 "arith_intensity_flop_per_byte": ai})

    # per-phase breakdown: three more runs outside the timed region, with every phase timed
    prm.timing_level = 0
    h_full = B.brsvd_create(prm)
    full = {}
    nb = 3
    for _ in range(nb):
        _, _, _, st = B.brsvd_run(h_full, A, Om, U, S, Vt, want_stats=True)
        for key, val in st.items():
            full[key] = full.get(key, 0) + val if key.endswith("seconds") else val
    B.brsvd_destroy(h_full)
    breakdown = {key: full[key] / nb * 1e3 for key in full if key.endswith("seconds")}
    breakdown["jacobi_sweeps"] = full["jacobi_sweeps"]
    breakdown["note"] = "untimed extra runs with every phase timed; the timed region times the pass kernels and the total"

    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import brsvd_oracle as O
        cores = len(os.sched_getaffinity(0))
        A_h = A.cpu().numpy()
        Om_h = Om.cpu().numpy()
        c0 = time.perf_counter()
        Uo, so, Vto = O.brsvd(A_h, Om_h, k, p, q, row_block=cfg.row_block)
        c1 = time.perf_counter()
        cpu_sec = c1 - c0
        cpu = {"value": bytes_a / cpu_sec / 1e9, "unit": "GB/s of A streamed", "cores": cores, "kind": "oracle",
               "seconds_per_brsvd": cpu_sec,
               "sample": f"one full fp64 BRSVD of the same {m}x{n} A and Omega (k={k}, p={p}, q={q})"}
        sg = S.double().cpu().numpy()
        parity = {"sigma_topk_max_rel": float(np.max(np.abs(sg[:k] - so[:k]) / so[:k]))}

    out = {
        "metric": "GB/s of A streamed per rank-k BRSVD (seconds per BRSVD in ms_per_step)",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "seconds_per_brsvd": sec, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name} in-core: A {'fp64' if f64 else 'fp32'} {m}x{n}, k={k}, p={p}, q={q}, row_block={cfg.row_block}, "
                               f"{passes} passes over A" + (" (fused)" if args.fused else ""), "m": m, "n": n, "k": k, "p": p, "q": q,
                   "row_block": cfg.row_block, "a_location": "device"},
        "roofline": roof, "cpu_baseline": cpu, "breakdown_ms": breakdown, "parity": parity,
    }
    B.brsvd_destroy(h)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
