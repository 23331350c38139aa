#!/usr/bin/env python3
"""Benchmark of the block randomized SVD hot path on one MI355X.

Headline (the timed region): a "step" is one complete rank-k BRSVD (all passes over A, orthonormalisations,
small SVD, lifts) of the largest in-core configuration, C3: A fp32 100000 x 50000 (20 GB, rank-512 Gaussian
factors, sigma_i = exp(-i/64), + 1e-5 noise), k = 256, p = 16, q = 1, row block 8192, with A and Omega resident
in HBM before the timed region.  Prints ONE JSON line: GB/s of A streamed per BRSVD (passes * 4*m*n bytes /
seconds), the roofline of the dominant kernel measured with HIP events inside the library, the fp64 CPU oracle
timed on this machine's host cores on a bounded sample, and -- measured after the timed region, in the same line
under "sub_records" -- the other named configurations:
  C2  in-core square 20000 x 20000, k = 100, p = 10, q = 2: ms per BRSVD and its dominant kernel;
  C5  robust PCA, 76800 x 2000, 30 ALM iterations with k = p = 10, q = 1: ms per iteration and the HBM fraction
      of the two pass kernels and of the fused update kernel;
  C4  out-of-core, A in pinned host memory streamed through two staging buffers under a 16 GB device budget:
      GB/s of A over the host link and its fraction of a plain pinned copy measured in the same run.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1|C2|C3] [--sub C2,C5,C4|none]
                  [--only C4|C5] [--no-cpu-baseline] [--fused] [--dtype f32|f64] [--copy-calibration] [--peaks]
  python bench.py --sweep gemm|shapes|rpca [--shape MxN ...] [--l L ...] [--family tall|square] [--gb G ...]
                  [--iters I] [--tol T] [--dtype f32|f64]      (kernel, shape and robust-PCA sweeps; JSON lines)
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
C4_ROWS = 160000              # the GPU machine pins at most about 64 GB of host memory: 160000 of the 200000 rows

# HBM bytes per launch of the pass kernels from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, each
# scaled by a plain 1 GiB copy in the same run.  Hardware counters cannot be read from inside the timed run, so
# these are offline figures; `traffic_source` in the JSON names the summary they come from.
OFFLINE_HBM_TRAFFIC = {
    "C3:gemm_an": 2.2266e10, "C3:gemm_at": 2.4204e10,
    "C2:gemm_an": 1.7246e9, "C2:gemm_at": 1.8517e9,
    "C5:gemm_an": 6.8064e8, "C5:gemm_at": 7.0227e8, "C5:rpca_update": 2.5175e9,
}
OFFLINE_HBM_TRAFFIC_SOURCE = {
    "C3:gemm_an": "profiles/gemm_thin_C3_hbm_traffic.md", "C3:gemm_at": "profiles/gemm_thin_C3_hbm_traffic.md",
    "C2:gemm_an": "profiles/gemm_thin_C2_hbm_traffic.md", "C2:gemm_at": "profiles/gemm_thin_C2_hbm_traffic.md",
    "C5:gemm_an": "profiles/gemm_thin_C5_hbm_traffic.md", "C5:gemm_at": "profiles/gemm_thin_C5_hbm_traffic.md",
    "C5:rpca_update": "profiles/gemm_thin_C5_hbm_traffic.md",
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def kernel_figures(m, n, l, esz, seconds, launches, peak_mfma):
    """Roofline figures of one pass kernel: algorithmic bytes 4mn + 4(m+n)l and flops 2mnl per launch over all of A."""
    avg = seconds / max(launches, 1)
    by = float(esz) * m * n + float(esz) * (m + n) * l
    fl = 2.0 * m * n * l
    return {"avg_launch_ms": avg * 1e3, "hbm_GBps": by / avg / 1e9, "hbm_frac": by / avg / 1e9 / PEAK_HBM_GBS,
            "mfma_TFLOPs": fl / avg / 1e12, "mfma_frac": fl / avg / 1e12 / peak_mfma,
            "algorithmic_bytes": by, "algorithmic_flops": fl}


def run_in_core(B, torch, cfg, steps, warmup, fused=False, f64=False, copy_calibration=False, breakdown_runs=3):
    """Times `steps` BRSVDs of an in-core configuration.  Returns (record, A, Om, S) with A, Om left on the device."""
    dev = torch.device("cuda:0")
    m, n, k, p, q, l = cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, cfg.l
    tdt = torch.float64 if f64 else torch.float32
    esz = 8 if f64 else 4
    A = cfg.make_A(device=dev)
    Om = cfg.make_Omega(device=dev)
    if f64:
        A, Om = A.double(), Om.double()
    torch.cuda.synchronize()
    prm = B.make_params(m, n, k, p, q, row_block=cfg.row_block,
                        pass_mode=B.BRSVD_PASSES_FUSED if fused else B.BRSVD_PASSES_SEPARATE,
                        dtype=B.BRSVD_DTYPE_F64 if f64 else B.BRSVD_DTYPE_F32,
                        timing_level=1)     # the timed region times the pass kernels and the total only
    h = B.brsvd_create(prm)
    U = torch.empty(m, l, device=dev, dtype=tdt)
    S = torch.empty(l, device=dev, dtype=tdt)
    Vt = torch.empty(l, n, device=dev, dtype=tdt)
    for _ in range(warmup):
        B.brsvd_run(h, A, Om, U, S, Vt, want_stats=False)
    torch.cuda.synchronize()
    if copy_calibration:
        src = torch.ones(1 << 28, device=dev)          # 1 GiB of fp32
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # timed region: exactly `steps` steps, statistics (HIP events inside the library) collected live
    acc = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        _, _, _, st = B.brsvd_run(h, A, Om, U, S, Vt, want_stats=True)
        for key, val in st.items():
            acc[key] = acc.get(key, 0) + val if key.endswith(("seconds", "launches", "_A", "streamed", "kernels")) else val
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.brsvd_destroy(h)
    sec = (t1 - t0) / steps
    passes = acc["passes_over_A"] // steps
    bytes_a = float(acc["bytes_A_streamed"]) / steps
    peak_mfma = PEAK_MFMA_F64_TFLOPS if f64 else PEAK_MFMA_F32_TFLOPS
    kern = {"gemm_an": kernel_figures(m, n, l, esz, acc["gemm_an_seconds"], acc["gemm_an_launches"], peak_mfma),
            "gemm_at": kernel_figures(m, n, l, esz, acc["gemm_at_seconds"], acc["gemm_at_launches"], peak_mfma)}
    kname = "gemm_an" if acc["gemm_an_seconds"] >= acc["gemm_at_seconds"] else "gemm_at"
    kf = kern[kname]
    ai = kf["algorithmic_flops"] / kf["algorithmic_bytes"]
    ridge = peak_mfma * 1e12 / (PEAK_HBM_GBS * 1e9)
    key = f"{cfg.name}:{kname}"
    traffic = None if (f64 or fused) else OFFLINE_HBM_TRAFFIC.get(key)
    if ai >= ridge:
        roof = {"bound": "mfma", "achieved": kf["mfma_TFLOPs"], "peak": peak_mfma, "unit": "TFLOP/s",
                "frac": kf["mfma_frac"], "traffic": traffic}
    else:
        roof = {"bound": "hbm", "achieved": kf["hbm_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": kf["hbm_frac"], "traffic": traffic}
    roof.update({"traffic_source": OFFLINE_HBM_TRAFFIC_SOURCE.get(key) if traffic else None,
                 "kernel": kname, "avg_launch_ms": kf["avg_launch_ms"], "launches_per_step": acc[f"{kname}_launches"] / steps,
                 "hbm_GBps": kf["hbm_GBps"], "hbm_frac": kf["hbm_frac"], "mfma_TFLOPs": kf["mfma_TFLOPs"],
                 "mfma_frac": kf["mfma_frac"], "arith_intensity_flop_per_byte": ai, "ridge_flop_per_byte": ridge,
                 "other_pass_kernel": {"kernel": "gemm_at" if kname == "gemm_an" else "gemm_an",
                                       **{k_: v for k_, v in kern["gemm_at" if kname == "gemm_an" else "gemm_an"].items()
                                          if not k_.startswith("algorithmic")}},
                 "split_sum_ms_per_step": acc["split_sum_seconds"] / steps * 1e3,
                 "note": "per-launch figures time the product kernels alone; the kernels that add the partial panels of "
                         "split launches are timed separately (split_sum_ms_per_step)"})

    # per-phase breakdown: further runs outside the timed region, with every phase timed
    breakdown = None
    if breakdown_runs:
        prm.timing_level = 0
        h_full = B.brsvd_create(prm)
        full = {}
        for _ in range(breakdown_runs):
            _, _, _, st = B.brsvd_run(h_full, A, Om, U, S, Vt, want_stats=True)
            for key, val in st.items():
                full[key] = full.get(key, 0) + val if key.endswith("seconds") else val
        B.brsvd_destroy(h_full)
        breakdown = {key: full[key] / breakdown_runs * 1e3 for key in full if key.endswith("seconds")}
        breakdown["jacobi_sweeps"] = full["jacobi_sweeps"]
        breakdown["note"] = "ms per BRSVD; untimed extra runs with every phase timed"
    rec = {"ms_per_brsvd": sec * 1e3, "A_GBps": bytes_a / sec / 1e9, "passes_over_A": passes, "bytes_A_per_brsvd": bytes_a,
           "gemm_TFLOPs_end_to_end": passes * 2.0 * m * n * l / sec / 1e12,
           "workload": f"{cfg.name} in-core: A {'fp64' if f64 else 'fp32'} {m}x{n}, k={k}, p={p}, q={q}, "
                       f"row_block={cfg.row_block}, {passes} passes over A" + (" (fused pass mode)" if fused else ""),
           "roofline": roof, "breakdown_ms": breakdown}
    del U, Vt
    return rec, A, Om, S


def oracle_baseline(np, A, Om, cfg, S, sample_rows, esz):
    """The fp64 oracle on the first `sample_rows` rows of the same A with the same Omega (all rows: the whole workload).
    Returns the cpu_baseline object and, when the sample is the whole matrix, the parity of the singular values."""
    from oracle import brsvd_oracle as O
    cores = len(os.sched_getaffinity(0))
    rows = min(sample_rows, cfg.m)
    A_h = A[:rows].cpu().numpy()
    Om_h = Om.cpu().numpy()
    c0 = time.perf_counter()
    Uo, so, Vto = O.brsvd(A_h, Om_h, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block)
    cpu_sec = time.perf_counter() - c0
    passes = 2 * cfg.q + 2
    whole = rows == cfg.m
    sample = (f"one full fp64 BRSVD of the same {cfg.m}x{cfg.n} A and Omega" if whole else
              f"one fp64 BRSVD of the first {rows} rows ({rows // cfg.row_block} row blocks of {cfg.row_block}) of the same "
              f"{cfg.m}x{cfg.n} A, all {cfg.n} columns, same Omega") + f" (k={cfg.k}, p={cfg.p}, q={cfg.q}, {passes} passes)"
    cpu = {"value": passes * float(esz) * rows * cfg.n / cpu_sec / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
           "seconds": cpu_sec, "sample": sample,
           "seconds_per_brsvd_extrapolated": cpu_sec * cfg.m / rows}
    parity = None
    if whole:
        sg = S.double().cpu().numpy()
        parity = {"sigma_topk_max_rel": float(np.max(np.abs(sg[:cfg.k] - so[:cfg.k]) / so[:cfg.k]))}
    return cpu, parity


def sub_c5(B, torch, np, synth, reps=3):
    """Robust PCA loop of configuration 5: 30 ALM iterations, k = p = 10, q = 1."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["C5"]
    m, n, l, iters = cfg.m, cfg.n, cfg.l, cfg.rpca["iters"]
    D, L0, S0 = synth.make_rpca(cfg, device=dev)
    Om = synth.rpca_omegas(cfg, n, iters, device=dev)
    lam = 1.0 / np.sqrt(max(m, n))
    x0 = synth.gaussian(n, 1, cfg.seed + 5, device=dev).reshape(-1).contiguous()
    h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block, timing_level=1))
    try:
        n2 = B.brsvd_norm2_power(h, D, x0, 20)
        L = torch.empty_like(D)
        S = torch.empty_like(D)
        work = torch.empty(2 * m * n, device=dev, dtype=D.dtype)
        best = None
        for _ in range(reps):
            L, S, res, st = B.brsvd_rpca_ialm(h, D, Om, iters, lam, 1.25 / n2, 1.5, norm2_M=n2, L=L, S=S, work=work)
            if best is None or st["total_seconds"] < best["total_seconds"]:
                best = st
    finally:
        B.brsvd_destroy(h)
    st = best
    an = kernel_figures(m, n, l, 4, st["gemm_an_seconds"], st["gemm_an_launches"], PEAK_MFMA_F32_TFLOPS)
    at = kernel_figures(m, n, l, 4, st["gemm_at_seconds"], st["gemm_at_launches"], PEAK_MFMA_F32_TFLOPS)
    upd = st["rpca_update_seconds"] / max(st["rpca_update_launches"], 1)
    upd_bytes = 16.0 * m * n          # reads M, Y; writes Y, X (L and S are formed once, after the loop)
    rec = {"workload": f"C5 robust PCA: D fp32 {m}x{n}, {iters} ALM iterations, k={cfg.k}, p={cfg.p}, q={cfg.q}, "
                       f"{st['passes_over_A'] // iters} passes over the iterate per iteration",
           "ms_per_iteration": st["total_seconds"] / iters * 1e3, "ms_total": st["total_seconds"] * 1e3,
           "bound": "hbm",
           "gemm_an": {"avg_launch_us": an["avg_launch_ms"] * 1e3, "hbm_GBps": an["hbm_GBps"], "hbm_frac": an["hbm_frac"],
                       "algorithmic_bytes": an["algorithmic_bytes"], "traffic": OFFLINE_HBM_TRAFFIC.get("C5:gemm_an")},
           "gemm_at": {"avg_launch_us": at["avg_launch_ms"] * 1e3, "hbm_GBps": at["hbm_GBps"], "hbm_frac": at["hbm_frac"],
                       "algorithmic_bytes": at["algorithmic_bytes"], "traffic": OFFLINE_HBM_TRAFFIC.get("C5:gemm_at")},
           "rpca_update": {"avg_launch_us": upd * 1e6, "hbm_GBps": upd_bytes / upd / 1e9,
                           "hbm_frac": upd_bytes / upd / 1e9 / PEAK_HBM_GBS, "algorithmic_bytes": upd_bytes,
                           "traffic": OFFLINE_HBM_TRAFFIC.get("C5:rpca_update")},
           "traffic_source": OFFLINE_HBM_TRAFFIC_SOURCE.get("C5:gemm_an"),
           "ms_per_iteration_by_phase": {key[:-8]: st[key] / iters * 1e3 for key in
                                         ("gemm_an_seconds", "gemm_at_seconds", "split_sum_seconds", "rpca_update_seconds")},
           "final_residual": res[-1],
           "L_vs_planted": float(torch.linalg.norm(L - L0) / torch.linalg.norm(L0)),
           "S_vs_planted": float(torch.linalg.norm(S - S0) / torch.linalg.norm(S0))}
    del D, L0, S0, Om, L, S, work
    return rec


def sub_c4(B, torch, synth, rows=C4_ROWS, reps=2):
    """Out-of-core configuration 4 at `rows` rows: host-link throughput against a plain pinned copy."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["C4"]
    if rows != cfg.m:
        cfg = cfg.scaled(rows, cfg.n)
    t0 = time.perf_counter()
    pm = B.PinnedMatrix(cfg.m, cfg.n)
    log(f"C4: pinned {4.0 * cfg.m * cfg.n / 1e9:.1f} GB in {time.perf_counter() - t0:.1f} s")
    try:
        t0 = time.perf_counter()
        cfg.make_A(device="cpu", out=pm.tensor, gen_device=dev)
        Om = cfg.make_Omega(device=dev)
        torch.cuda.synchronize()
        log(f"C4: generated A in {time.perf_counter() - t0:.1f} s")
        blk = torch.empty(cfg.row_block, cfg.n, device=dev)
        h2d = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            blk.copy_(pm.tensor[:cfg.row_block], non_blocking=True)
            e1.record()
            torch.cuda.synchronize()
            h2d = max(h2d, blk.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del blk
        prm = B.make_params(cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block, a_location=B.BRSVD_A_HOST_PINNED,
                            device_budget_bytes=cfg.device_budget, timing_level=1)
        ws_bytes = B.brsvd_workspace_bytes(prm)
        h = B.brsvd_create(prm)
        try:
            best = None
            for i in range(reps):
                U, S, Vt, st = B.brsvd_run(h, pm.tensor, Om, pinned=True)
                log(f"C4: run {i}: {st['total_seconds']:.3f} s")
                if best is None or st["total_seconds"] < best["total_seconds"]:
                    best = st
        finally:
            B.brsvd_destroy(h)
        t = best["total_seconds"]
        eye = torch.eye(cfg.l, device=dev, dtype=torch.float64)
        orth = float(torch.linalg.matrix_norm(U.double().T @ U.double() - eye, 2))
        link = best["bytes_A_streamed"] / t / 1e9
        return {"workload": f"C4 out-of-core: A fp32 {cfg.m}x{cfg.n} ({4.0 * cfg.m * cfg.n / 1e9:.0f} GB) in pinned host memory, "
                            f"k={cfg.k}, p={cfg.p}, q={cfg.q}, row_block={cfg.row_block}, two staging buffers, device budget "
                            f"{cfg.device_budget / 2 ** 30:.0f} GiB; the configuration names 200000 rows (80 GB), the box pins "
                            f"at most about 64 GB",
                "bound": "host link", "seconds_per_brsvd": t, "passes_over_A": best["passes_over_A"], "blocks": best["n_blocks"],
                "workspace_GB": ws_bytes / 1e9, "link_GBps": link, "pinned_copy_GBps": h2d,
                "frac_of_pinned_copy": link / h2d, "copy_seconds": best["copy_seconds"],
                "gemm_seconds": best["gemm_an_seconds"] + best["gemm_at_seconds"],
                "bytes_A_read_by_kernels_GB": best["bytes_A_read_by_kernels"] / 1e9, "orth_defect_U": orth}
    finally:
        pm.free()


def measured_peaks(B, torch):
    dev = torch.device("cuda:0")
    buf = torch.randn(1 << 30, device=dev)                 # 4 GiB of fp32
    sec, work = B.brsvd_probe(0, buf, buf.numel() * 4)
    out = {"hbm_streaming_read_GBps": work / sec / 1e9}
    del buf
    o = torch.empty(2048 * 256, device=dev)
    sec, work = B.brsvd_probe(1, o, 20000)
    out["mfma_f32_TFLOPs"] = work / sec / 1e12
    return out


# ---- sweeps (not part of the default run; every line of output is one JSON object) ----------------------------
def _time_ms(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def sweep_gemm(B, torch, args):
    """The two pass kernels alone (HIP events inside the library around the product kernels of one BRSVD with q = 1):
    microseconds, Tflop/s and GB/s of the algorithmic bytes 4mn + 4(m+n)l.  l <= 32 is the HBM-bound side of the ridge."""
    dev = torch.device("cuda:0")
    for shape in args.shape or ["20000x20000", "100000x50000"]:
        m, n = (int(x) for x in shape.lower().split("x"))
        A = torch.randn(m, n, device=dev)
        for l in args.l or [8, 16, 32, 64, 110, 272]:
            Om = torch.randn(n, l, device=dev)
            h = B.brsvd_create(B.make_params(m, n, l, 0, 1, row_block=0, timing_level=1))
            best = None
            try:
                for _ in range(4):
                    _, _, _, st = B.brsvd_run(h, A, Om)
                    t = st["gemm_an_seconds"] + st["gemm_at_seconds"]
                    if best is None or t < best["gemm_an_seconds"] + best["gemm_at_seconds"]:
                        best = st
            finally:
                B.brsvd_destroy(h)
            rec = {"m": m, "n": n, "l": l}
            for name in ("gemm_an", "gemm_at"):
                f = kernel_figures(m, n, l, 4, best[f"{name}_seconds"], best[f"{name}_launches"], PEAK_MFMA_F32_TFLOPS)
                rec[name] = {"us": round(f["avg_launch_ms"] * 1e3, 1), "GBps": round(f["hbm_GBps"]), "hbm_frac": round(f["hbm_frac"], 3),
                             "TFLOPs": round(f["mfma_TFLOPs"], 1), "mfma_frac": round(f["mfma_frac"], 3)}
            print(json.dumps(rec), flush=True)
        del A


def sweep_shapes(B, torch, args):
    """Whole rank-k BRSVDs over growing inputs at the two aspect ratios of the paper's Fig. 2 (tall-skinny m:n:k =
    1024:32:1, square 256:256:1; rank-k Gaussian-product inputs as in Sec. 4, p = 10, q = 1): seconds, Tflop/s with the
    flop count of the paper's Table 1 terms written out, and the share of each phase."""
    dev = torch.device("cuda:0")
    fams = {"tall": (1024, 32), "square": (256, 256)}
    f64 = args.dtype == "f64"
    tdt, esz = (torch.float64, 8) if f64 else (torch.float32, 4)
    p, q = 10, 1
    for fam in args.family or ["tall", "square"]:
        rm, rn = fams[fam]
        for gb in args.gb or [0.25, 1, 4, 16]:
            k = max(2, int(round((gb * 1e9 / esz / (rm * rn)) ** 0.5)))
            m, n, l = rm * k, rn * k, k + p
            if l > min(m, n, 512):
                print(json.dumps({"family": fam, "gb": gb, "skipped": f"l = {l} exceeds min(m, n, 512)"}), flush=True)
                continue
            g = torch.Generator(device=dev)
            g.manual_seed(1000 + k)
            A = torch.empty(m, n, device=dev, dtype=tdt)
            G2 = torch.randn(k, n, device=dev, generator=g, dtype=tdt)
            step = max(1, (1 << 27) // max(n, 1))
            for r0 in range(0, m, step):
                r1 = min(m, r0 + step)
                A[r0:r1] = torch.randn(r1 - r0, k, device=dev, generator=g, dtype=tdt) @ G2
            Om = torch.randn(n, l, device=dev, dtype=tdt)
            h = B.brsvd_create(B.make_params(m, n, k, p, q, row_block=0, dtype=B.BRSVD_DTYPE_F64 if f64 else B.BRSVD_DTYPE_F32))
            try:
                B.brsvd_run(h, A, Om, want_stats=False)
                best = None
                for _ in range(3):
                    U, S, Vt, st = B.brsvd_run(h, A, Om)
                    if best is None or st["total_seconds"] < best["total_seconds"]:
                        best = st
            finally:
                B.brsvd_destroy(h)
            sweeps = (q + 1) + q + 4           # one CholeskyQR sweep per intermediate panel, two per output basis
            flops = 2.0 * m * n * l * (2 * q + 2) + 2.0 * (m + n) * l * l * (sweeps + 1)
            t = best["total_seconds"]
            err = float(torch.linalg.norm(A[:4096] - (U[:4096] * S) @ Vt) / torch.linalg.norm(A[:4096]))
            print(json.dumps({"family": fam, "dtype": args.dtype, "m": m, "n": n, "k": k, "p": p, "q": q,
                              "bytes_A_GB": round(float(esz) * m * n / 1e9, 3), "seconds": round(t, 6),
                              "tflops": round(flops / t / 1e12, 2), "A_GBps": round(best["bytes_A_streamed"] / t / 1e9, 1),
                              "share": {key[:-8]: round(best[key] / t, 3) for key in
                                        ("gemm_an_seconds", "gemm_at_seconds", "orth_seconds", "svd_seconds", "lift_seconds")},
                              "orth_fallbacks": best["orth_fallbacks"], "rel_error_first_4096_rows": err}), flush=True)
            del A, Om, U, S, Vt


def sweep_rpca(B, torch, np, synth, args):
    """Alg. 3 with its stopping rule (k = p = 10, q = 1) on synthetic rank-5 + 5 % sparse matrices of the shapes of the
    paper's Table 2 (and configuration 5): iterations, seconds, per-iteration milliseconds of the phases and the GB/s of
    the pass and update kernels."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["C5"]
    f64 = args.dtype == "f64"
    esz = 8 if f64 else 4
    for shape in args.shape or ["76800x2000", "2073600x100", "32256x2383"]:
        m, n = (int(x) for x in shape.lower().split("x"))
        D, L0, S0 = synth.make_rpca(cfg, device=dev, m=m, n=n)
        Om = synth.rpca_omegas(cfg, n, args.iters, device=dev)
        lam = 1.0 / np.sqrt(max(m, n))
        x0 = synth.gaussian(n, 1, cfg.seed + 5, device=dev).reshape(-1).contiguous()
        if f64:
            D, L0, S0, Om, x0 = D.double(), L0.double(), S0.double(), Om.double(), x0.double()
        h = B.brsvd_create(B.make_params(m, n, cfg.k, cfg.p, cfg.q, row_block=min(m, 65536),
                                         dtype=B.BRSVD_DTYPE_F64 if f64 else B.BRSVD_DTYPE_F32))
        try:
            n2 = B.brsvd_norm2_power(h, D, x0, 20)
            L, S = torch.empty_like(D), torch.empty_like(D)
            work = torch.empty(2 * m * n, device=dev, dtype=D.dtype)
            for _ in range(2):
                L, S, res, done, st = B.brsvd_rpca_ialm_tol(h, D, Om, args.iters, args.tol, lam, 1.25 / n2, 1.5,
                                                            norm2_M=n2, L=L, S=S, work=work)
        finally:
            B.brsvd_destroy(h)
        by = float(esz) * m * n
        an = st["gemm_an_seconds"] / max(st["gemm_an_launches"], 1)
        at = st["gemm_at_seconds"] / max(st["gemm_at_launches"], 1)
        up = st["rpca_update_seconds"] / max(st["rpca_update_launches"], 1)
        print(json.dumps({"m": m, "n": n, "dtype": args.dtype, "iterations": done, "tol": args.tol, "residual": res[-1],
                          "seconds": round(st["total_seconds"], 6),
                          "ms_per_iteration": {key[:-8]: round(st[key] / done * 1e3, 4) for key in
                                               ("total_seconds", "gemm_an_seconds", "gemm_at_seconds", "split_sum_seconds",
                                                "orth_seconds", "svd_seconds", "lift_seconds", "elementwise_seconds")},
                          "gemm_an_GBps": round(by / an / 1e9, 1), "gemm_at_GBps": round(by / at / 1e9, 1),
                          "rpca_update_GBps": round(4.0 * by / up / 1e9, 1),
                          "L_vs_planted": float(torch.linalg.norm(L - L0) / torch.linalg.norm(L0)),
                          "S_vs_planted": float(torch.linalg.norm(S - S0) / torch.linalg.norm(S0))}), flush=True)
        del D, L0, S0, Om, L, S, work


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", "--config", dest="workload", default="C3", choices=["C1", "C2", "C3"])
    ap.add_argument("--sub", default="C2,C5,C4", help="sub-records measured after the timed region (comma list, or none)")
    ap.add_argument("--only", default=None, choices=["C4", "C5"],
                    help="measure just this sub-record and print it as the JSON line (for profiler runs)")
    ap.add_argument("--c4-rows", type=int, default=C4_ROWS)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused", action="store_true",
                    help="fused pass mode instead of the 2q+2 separate passes the headline metric is quoted on")
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"],
                    help="f64 runs the same workload in double precision (brsvd_run_f64); the headline metric is f32")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (outside the timed region) so that a rocprofv3 "
                         "--pmc run has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    ap.add_argument("--peaks", action="store_true", help="add the measured streaming-read and fp32 MFMA peaks of this device")
    ap.add_argument("--sweep", default=None, choices=["gemm", "shapes", "rpca"],
                    help="instead of the benchmark line: the pass kernels over shapes and widths (gemm), whole BRSVDs at the "
                         "aspect ratios of the paper's Fig. 2 (shapes), or Alg. 3 at the shapes of its Table 2 (rpca)")
    ap.add_argument("--shape", nargs="+", default=None, help="sweeps gemm, rpca: MxN ...")
    ap.add_argument("--l", nargs="+", type=int, default=None, help="sweep gemm: sketch widths")
    ap.add_argument("--family", nargs="+", default=None, choices=["tall", "square"], help="sweep shapes")
    ap.add_argument("--gb", nargs="+", type=float, default=None, help="sweep shapes: input sizes in GB")
    ap.add_argument("--iters", type=int, default=30, help="sweep rpca: iteration cap")
    ap.add_argument("--tol", type=float, default=1e-7, help="sweep rpca: stopping tolerance")
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

    if args.sweep:
        if args.sweep == "gemm":
            sweep_gemm(B, torch, args)
        elif args.sweep == "shapes":
            sweep_shapes(B, torch, args)
        else:
            sweep_rpca(B, torch, np, synth, args)
        return 0

    if args.only:
        if args.copy_calibration:
            src = torch.ones(1 << 28, device="cuda:0")
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        rec = sub_c5(B, torch, np, synth) if args.only == "C5" else sub_c4(B, torch, synth, rows=args.c4_rows)
        print(json.dumps({"sub_record": args.only, **rec}))
        return 0

    f64 = args.dtype == "f64"
    esz = 8 if f64 else 4
    cfg = synth.CONFIGS[args.workload]
    t_start = time.perf_counter()
    rec, A, Om, S = run_in_core(B, torch, cfg, args.steps, args.warmup, fused=args.fused, f64=f64,
                                copy_calibration=args.copy_calibration)
    log(f"{cfg.name}: {rec['ms_per_brsvd']:.3f} ms per BRSVD ({time.perf_counter() - t_start:.1f} s)")

    cpu = parity = None
    if not args.no_cpu_baseline:
        # bounded sample: the whole workload where the oracle takes seconds, six row blocks of C3 (about 10 s)
        sample_rows = cfg.m if cfg.m * cfg.n <= 5e8 else 6 * cfg.row_block
        cpu, parity = oracle_baseline(np, A, Om, cfg, S, sample_rows, esz)
        log(f"oracle sample: {cpu['seconds']:.1f} s")
    del A, Om, S
    torch.cuda.empty_cache()

    subs = {}
    wanted = [] if args.sub.lower() == "none" else [s.strip().upper() for s in args.sub.split(",") if s.strip()]
    if any(name not in ("C1", "C2", "C3", "C4", "C5") for name in wanted):
        print(f"bench.py: unknown sub-record in {args.sub}", file=sys.stderr)
        return 2

    def c2_record():
        r, a_, o_, s_ = run_in_core(B, torch, synth.CONFIGS["C2"], 10, 2)
        del a_, o_, s_
        return r

    def c4_record():
        # a box that cannot pin the requested size still reports the recipe, at half the rows
        for rows in (args.c4_rows, args.c4_rows // 2):
            try:
                return sub_c4(B, torch, synth, rows=rows)
            except MemoryError as e:
                log(f"C4 at {rows} rows: {e}")
        raise MemoryError(f"cannot pin {args.c4_rows // 2} rows of C4 on this box")

    makers = {"C2": c2_record, "C5": lambda: sub_c5(B, torch, np, synth), "C4": c4_record}
    for name in wanted:
        t0 = time.perf_counter()
        if name == cfg.name or name not in makers:
            continue
        try:                                   # the headline line is printed whatever happens to a sub-record
            subs[name] = makers[name]()
        except Exception as e:                 # noqa: BLE001 -- recorded in the line, not swallowed
            subs[name] = {"error": f"{type(e).__name__}: {e}"}
            log(f"sub-record {name} failed: {subs[name]['error']}")
        torch.cuda.empty_cache()
        log(f"sub-record {name}: {time.perf_counter() - t0:.1f} s")

    out = {
        "metric": "GB/s of A streamed per rank-k BRSVD (seconds per BRSVD in ms_per_step)",
        "value": rec["A_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_brsvd"], "seconds_per_brsvd": rec["ms_per_brsvd"] * 1e-3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": rec["workload"], "m": cfg.m, "n": cfg.n, "k": cfg.k, "p": cfg.p, "q": cfg.q,
                   "row_block": cfg.row_block, "a_location": "device"},
        "roofline": rec["roofline"], "cpu_baseline": cpu, "breakdown_ms": rec["breakdown_ms"], "parity": parity,
        "gemm_TFLOPs_end_to_end": rec["gemm_TFLOPs_end_to_end"],
        "sub_records": subs,
    }
    if args.peaks:
        out["measured_peaks"] = measured_peaks(B, torch)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
