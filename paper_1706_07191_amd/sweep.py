"""Timing sweeps of the HIP path on one MI355X (synthetic Gaussian-product inputs, A resident in HBM).

  python -m paper_1706_07191_amd.sweep gemm   [--shape MxN ...] [--l L ...]
      the two pass kernels alone, one launch over all of A: ms, Tflop/s and GB/s of the algorithmic
      bytes 4*m*n + 4*(m+n)*l.  Narrow panels (l <= 32) are the HBM-bound side of the ridge.
  python -m paper_1706_07191_amd.sweep shapes [--family tall|square] [--gb G ...] [--q Q] [--p P] [--dtype f32|f64]
      whole rank-k BRSVDs over growing inputs at the two aspect ratios of the paper's Fig. 2
      (tall-skinny m:n:k = 1024:32:1, square m:n:k = 256:256:1): seconds, Tflop/s with the flop
      count of the paper's Table 1 terms written out, 2*m*n*l*(2q+2) for the passes plus
      2*(m+n)*l^2 per orthonormalisation sweep and lift, and the share of each phase.

  python -m paper_1706_07191_amd.sweep rpca   [--shape MxN ...] [--iters I] [--tol T] [--dtype f32|f64]
      the robust-PCA loop (Alg. 3, k = p = 10, q = 1) on a synthetic rank-5 + 5 % sparse matrix of the
      given shape (default: configuration 5 and the two shapes of the paper's Table 2): iterations,
      seconds, per-phase milliseconds per iteration and the GB/s of the pass and elementwise kernels.

  python -m paper_1706_07191_amd.sweep stream [--rows M] [--modes separate fused alg2]
      configuration 4 (A fp32 M x 100000 in pinned host memory, k = 128, p = 16, q = 1, blocks of 16384 rows
      through two staging buffers, 16 GB device budget): seconds per BRSVD, GB/s of A over the host link and the
      fraction of a plain pinned copy of one block measured in the same run.  M defaults to 160000 (64 GB).

  python -m paper_1706_07191_amd.sweep peaks
      measured peaks of this device next to the published ones: streaming read of 8 GiB of HBM, an fp32
      MFMA loop, a pinned host-to-device copy of 1 GiB.

Every line of output is one JSON object.
"""
from __future__ import annotations

import argparse
import json
import sys


def _time_ms(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _gaussian_product(m, n, r, dev, seed, dtype):
    import torch
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    A = torch.empty(m, n, device=dev, dtype=dtype)
    G2 = torch.randn(r, n, device=dev, generator=g, dtype=dtype)
    step = max(1, (1 << 27) // max(n, 1))
    for r0 in range(0, m, step):
        r1 = min(m, r0 + step)
        A[r0:r1] = torch.randn(r1 - r0, r, device=dev, generator=g, dtype=dtype) @ G2
    return A


def sweep_gemm(args):
    import torch

    import paper_1706_07191_amd as B
    dev = torch.device("cuda:0")
    for shape in args.shape:
        m, n = (int(x) for x in shape.lower().split("x"))
        A = torch.randn(m, n, device=dev)
        for l in args.l:
            X = torch.randn(n, l, device=dev)
            Q = torch.randn(m, l, device=dev)
            Y = torch.empty(m, l, device=dev)
            Z = torch.zeros(n, l, device=dev)
            by = 4.0 * m * n + 4.0 * (m + n) * l
            for name, fn in (("gemm_an", lambda: B.brsvd_gemm_an(A, X, Y)), ("gemm_at", lambda: B.brsvd_gemm_at(A, Q, Z))):
                ms = _time_ms(fn, args.reps)
                print(json.dumps({"kernel": name, "m": m, "n": n, "l": l, "ms": round(ms, 4),
                                  "tflops": round(2.0 * m * n * l / ms / 1e9, 2),
                                  "algorithmic_GBps": round(by / ms / 1e6, 1),
                                  "note": "includes the panel pad/unpad and split-sum kernels of the step-level call"}),
                      flush=True)
        del A


def sweep_shapes(args):
    import torch

    import paper_1706_07191_amd as B
    dev = torch.device("cuda:0")
    fams = {"tall": (1024, 32), "square": (256, 256)}
    f64 = args.dtype == "f64"
    tdt, esz = (torch.float64, 8) if f64 else (torch.float32, 4)
    for fam in args.family:
        rm, rn = fams[fam]
        for gb in args.gb:
            # m = rm*k, n = rn*k with esz*m*n = gb * 1e9 bytes
            k = max(2, int(round((gb * 1e9 / esz / (rm * rn)) ** 0.5)))
            m, n, p, q = rm * k, rn * k, args.p, args.q
            l = k + p
            if l > min(m, n, 512):
                print(json.dumps({"family": fam, "gb": gb, "skipped": f"l = {l} exceeds min(m, n, 512)"}), flush=True)
                continue
            A = _gaussian_product(m, n, k, dev, 1000 + k, tdt)
            Om = torch.randn(n, l, device=dev, dtype=tdt)
            h = B.brsvd_create(B.make_params(m, n, k, p, q, row_block=0,
                                             dtype=B.BRSVD_DTYPE_F64 if f64 else B.BRSVD_DTYPE_F32))
            try:
                B.brsvd_run(h, A, Om, want_stats=False)
                best = None
                for _ in range(args.reps):
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
                              "bytes_A_GB": round(float(esz) * m * n / 1e9, 3),
                              "seconds": round(t, 6), "tflops": round(flops / t / 1e12, 2),
                              "A_GBps": round(best["bytes_A_streamed"] / t / 1e9, 1),
                              "share": {key[:-8]: round(best[key] / t, 3) for key in
                                        ("gemm_an_seconds", "gemm_at_seconds", "orth_seconds", "svd_seconds", "lift_seconds")},
                              "orth_fallbacks": best["orth_fallbacks"], "passes_over_A": best["passes_over_A"],
                              "rel_error_first_4096_rows": err}), flush=True)
            del A, Om, U, S, Vt


def sweep_rpca(args):
    import numpy as np
    import torch

    import paper_1706_07191_amd as B
    from paper_1706_07191_amd import synth
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["C5"]
    f64 = args.dtype == "f64"
    esz = 8 if f64 else 4
    for shape in args.shape:
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
            L = torch.empty_like(D)
            S = torch.empty_like(D)
            work = torch.empty(2 * m * n, device=dev, dtype=D.dtype)
            for _ in range(args.reps):
                L, S, res, done, st = B.brsvd_rpca_ialm_tol(h, D, Om, args.iters, args.tol, lam, 1.25 / n2, 1.5,
                                                            norm2_M=n2, L=L, S=S, work=work)
        finally:
            B.brsvd_destroy(h)
        by = float(esz) * m * n
        an = st["gemm_an_seconds"] / max(st["gemm_an_launches"], 1)
        at = st["gemm_at_seconds"] / max(st["gemm_at_launches"], 1)
        print(json.dumps({"m": m, "n": n, "dtype": args.dtype, "iterations": done, "tol": args.tol, "residual": res[-1],
                          "seconds": round(st["total_seconds"], 6),
                          "ms_per_iteration": {key[:-8]: round(st[key] / done * 1e3, 4) for key in
                                               ("total_seconds", "gemm_an_seconds", "gemm_at_seconds", "orth_seconds",
                                                "svd_seconds", "lift_seconds", "elementwise_seconds")},
                          "gemm_an_GBps": round(by / an / 1e9, 1), "gemm_at_GBps": round(by / at / 1e9, 1),
                          "elementwise_GBps": round(5.0 * esz * m * n / (st["elementwise_seconds"] / done) / 1e9, 1),
                          "L_vs_planted": float(torch.linalg.norm(L - L0) / torch.linalg.norm(L0)),
                          "S_vs_planted": float(torch.linalg.norm(S - S0) / torch.linalg.norm(S0))}), flush=True)
        del D, L0, S0, Om, L, S, work


def sweep_stream(args):
    import torch

    import paper_1706_07191_amd as B
    from paper_1706_07191_amd import synth
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["C4"]
    if args.rows != cfg.m:
        cfg = cfg.scaled(args.rows, cfg.n)
    pm = B.PinnedMatrix(cfg.m, cfg.n)
    Ap = pm.tensor
    cfg.make_A(device="cpu", out=Ap, gen_device=dev)
    Om = cfg.make_Omega(device=dev)
    blk = torch.empty(cfg.row_block, cfg.n, device=dev)
    h2d = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        blk.copy_(Ap[:cfg.row_block], non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        h2d = max(h2d, blk.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del blk
    for mode in args.modes:
        prm = B.make_params(cfg.m, cfg.n, cfg.k, cfg.p, cfg.q, row_block=cfg.row_block, a_location=B.BRSVD_A_HOST_PINNED,
                            device_budget_bytes=cfg.device_budget,
                            pass_mode=B.BRSVD_PASSES_FUSED if mode == "fused" else B.BRSVD_PASSES_SEPARATE)
        h = B.brsvd_create(prm)
        try:
            best = None
            for _ in range(args.reps):
                if mode == "alg2":
                    U, S, Vt, st = B.brsvd_run_alg2(h, Ap, cfg.l, seed=777, pinned=True)
                else:
                    U, S, Vt, st = B.brsvd_run(h, Ap, Om, pinned=True)
                if best is None or st["total_seconds"] < best["total_seconds"]:
                    best = st
        finally:
            B.brsvd_destroy(h)
        t = best["total_seconds"]
        orth = float(torch.linalg.matrix_norm(U.double().T @ U.double() - torch.eye(cfg.l, device=dev, dtype=torch.float64), 2))
        print(json.dumps({"mode": mode, "m": cfg.m, "n": cfg.n, "l": cfg.l, "bytes_A_GB": round(4.0 * cfg.m * cfg.n / 1e9, 1),
                          "workspace_GB": round(B.brsvd_workspace_bytes(prm) / 1e9, 2), "blocks": best["n_blocks"],
                          "passes": best["passes_over_A"], "seconds": round(t, 4),
                          "link_GBps": round(best["bytes_A_streamed"] / t / 1e9, 2), "pinned_copy_GBps": round(h2d, 2),
                          "fraction_of_pinned_copy": round(best["bytes_A_streamed"] / t / 1e9 / h2d, 4),
                          "copy_seconds": round(best["copy_seconds"], 4),
                          "gemm_seconds": round(best["gemm_an_seconds"] + best["gemm_at_seconds"], 4),
                          "orthU": orth}), flush=True)
        del U, S, Vt


def sweep_peaks(args):
    import torch

    import paper_1706_07191_amd as B
    dev = torch.device("cuda:0")
    buf = torch.randn(1 << 31, device=dev)                 # 8 GiB of fp32
    sec, work = B.brsvd_probe(0, buf, buf.numel() * 4)
    print(json.dumps({"probe": "hbm streaming read", "GBps": round(work / sec / 1e9, 1), "published_GBps": 8000}), flush=True)
    del buf
    out = torch.empty(2048 * 256, device=dev)
    sec, work = B.brsvd_probe(1, out, 20000)
    print(json.dumps({"probe": "fp32 MFMA 16x16x4, random operands", "TFLOPs": round(work / sec / 1e12, 1),
                      "published_TFLOPs": 157.3}), flush=True)
    host = torch.empty(1 << 28, dtype=torch.float32, pin_memory=True)
    d = torch.empty(1 << 28, device=dev)
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        d.copy_(host, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, d.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    print(json.dumps({"probe": "pinned host-to-device copy of 1 GiB", "GBps": round(best, 1)}), flush=True)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    g = sub.add_parser("gemm")
    g.add_argument("--shape", nargs="+", default=["20000x20000", "100000x50000"])
    g.add_argument("--l", nargs="+", type=int, default=[8, 16, 32, 64, 110, 272])
    g.add_argument("--reps", type=int, default=5)
    s = sub.add_parser("shapes")
    s.add_argument("--family", nargs="+", default=["tall", "square"], choices=["tall", "square"])
    s.add_argument("--gb", nargs="+", type=float, default=[0.25, 1, 4, 16])
    s.add_argument("--p", type=int, default=10)
    s.add_argument("--q", type=int, default=1)
    s.add_argument("--reps", type=int, default=3)
    s.add_argument("--dtype", default="f32", choices=["f32", "f64"])
    r = sub.add_parser("rpca")
    r.add_argument("--shape", nargs="+", default=["76800x2000", "2073600x100", "32256x2383"])
    r.add_argument("--iters", type=int, default=30)
    r.add_argument("--tol", type=float, default=1e-7)
    r.add_argument("--reps", type=int, default=2)
    r.add_argument("--dtype", default="f32", choices=["f32", "f64"])
    sub.add_parser("peaks")
    t = sub.add_parser("stream")
    t.add_argument("--rows", type=int, default=160000)
    t.add_argument("--modes", nargs="+", default=["separate", "fused", "alg2"], choices=["separate", "fused", "alg2"])
    t.add_argument("--reps", type=int, default=2)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 2
    import paper_1706_07191_amd as B
    B.lib()
    {"gemm": sweep_gemm, "shapes": sweep_shapes, "rpca": sweep_rpca, "stream": sweep_stream, "peaks": sweep_peaks}[args.cmd](args)
    return 0


if __name__ == "__main__":
    sys.exit(main())
