"""Thin ctypes binding of libbrsvd (hand-written HIP for MI355X / gfx950).

Only argument marshalling lives here: torch provides device memory and streams, every step of
the block randomized SVD runs inside the shared library.  The functions carry the same names
as the C entry points declared in include/brsvd.h.  There is no CPU fallback: if the shared
library has not been built (python -m paper_1706_07191_amd.build) importing `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbrsvd.so")

BRSVD_OK = 0
BRSVD_ERR_ARG = -1
BRSVD_ERR_BUDGET = -2
BRSVD_ERR_ALLOC = -3
BRSVD_ERR_HIP = -4
BRSVD_ERR_ORTH_BREAKDOWN = -5
BRSVD_ERR_SVD_NOCONV = -6
BRSVD_A_DEVICE = 0
BRSVD_A_HOST_PINNED = 1
BRSVD_ORTH_AUTO = 0
BRSVD_ORTH_CHOLQR2 = 1
BRSVD_ORTH_TSQR = 2
BRSVD_PASSES_SEPARATE = 0
BRSVD_PASSES_FUSED = 1
BRSVD_DTYPE_F32 = 0
BRSVD_DTYPE_F64 = 1


class brsvd_params(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64),
                ("k", C.c_int32), ("p", C.c_int32), ("q", C.c_int32), ("a_location", C.c_int32),
                ("row_block", C.c_int64), ("device_budget_bytes", C.c_uint64),
                ("orth_method", C.c_int32), ("pass_mode", C.c_int32),
                ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p),
                ("dtype", C.c_int32), ("timing_level", C.c_int32),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64)]


class brsvd_stats(C.Structure):
    _fields_ = [("total_seconds", C.c_double), ("gemm_an_seconds", C.c_double),
                ("gemm_at_seconds", C.c_double), ("orth_seconds", C.c_double),
                ("svd_seconds", C.c_double), ("lift_seconds", C.c_double),
                ("copy_seconds", C.c_double), ("elementwise_seconds", C.c_double),
                ("gemm_an_launches", C.c_int64), ("gemm_at_launches", C.c_int64),
                ("passes_over_A", C.c_int64), ("bytes_A_streamed", C.c_int64),
                ("orth_fallbacks", C.c_int32), ("jacobi_sweeps", C.c_int32),
                ("row_block", C.c_int32), ("n_blocks", C.c_int32),
                ("split_sum_seconds", C.c_double), ("rpca_update_seconds", C.c_double),
                ("rpca_update_launches", C.c_int64), ("bytes_A_read_by_kernels", C.c_int64),
                ("fused_fallbacks", C.c_int32), ("reserved_", C.c_int32)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


# entry points declared in include/brsvd.h (the product calls) and include/brsvd_steps.h (the steps)
EXPORTS = ["brsvd_workspace_bytes", "brsvd_create", "brsvd_run", "brsvd_run_f64", "brsvd_rpca_ialm",
           "brsvd_rpca_ialm_tol", "brsvd_rpca_ialm_tol_f64", "brsvd_norm2_power", "brsvd_norm2_power_f64",
           "brsvd_run_alg2", "brsvd_run_alg2_f64", "brsvd_philox_normal", "brsvd_philox_normal_f64",
           "brsvd_destroy", "brsvd_status_string"]
STEP_EXPORTS = ["brsvd_gemm_an", "brsvd_gemm_at", "brsvd_gemm_scratch_bytes", "brsvd_gemm_an_f64",
                "brsvd_gemm_at_f64", "brsvd_gemm_scratch_bytes_f64", "brsvd_orth", "brsvd_orth_scratch_bytes",
                "brsvd_small_svd", "brsvd_small_svd_scratch_bytes", "brsvd_small_svd_static", "brsvd_gemm_plan",
                "brsvd_probe"]

_lib = None


class BrsvdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where} failed: {status} ({brsvd_status_string(status)})")


def lib() -> C.CDLL:
    """Loads libbrsvd.so (raises if it was not built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1706_07191_amd.build`; "
                          "there is no fallback implementation")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, dbl, flt = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_double, C.c_float
    L.brsvd_workspace_bytes.argtypes = [C.POINTER(brsvd_params), C.POINTER(u64)]
    L.brsvd_create.argtypes = [C.POINTER(brsvd_params), C.POINTER(vp)]
    L.brsvd_run.argtypes = [vp, vp, i64, vp, vp, vp, vp, C.POINTER(brsvd_stats)]
    L.brsvd_run_f64.argtypes = L.brsvd_run.argtypes
    L.brsvd_rpca_ialm.argtypes = [vp, vp, vp, i32, flt, flt, flt, dbl, vp, vp, vp, C.POINTER(dbl),
                                  C.POINTER(brsvd_stats)]
    L.brsvd_rpca_ialm_tol.argtypes = [vp, vp, vp, i32, dbl, flt, flt, flt, dbl, vp, vp, vp, C.POINTER(dbl),
                                      C.POINTER(i32), C.POINTER(brsvd_stats)]
    L.brsvd_rpca_ialm_tol_f64.argtypes = [vp, vp, vp, i32, dbl, dbl, dbl, dbl, dbl, vp, vp, vp, C.POINTER(dbl),
                                          C.POINTER(i32), C.POINTER(brsvd_stats)]
    L.brsvd_norm2_power.argtypes = [vp, vp, i64, vp, i32, C.POINTER(dbl)]
    L.brsvd_norm2_power_f64.argtypes = L.brsvd_norm2_power.argtypes
    L.brsvd_run_alg2.argtypes = [vp, vp, i64, u64, vp, vp, vp, vp, C.POINTER(brsvd_stats)]
    L.brsvd_philox_normal.argtypes = [u64, i64, i64, i32, vp, vp]
    L.brsvd_run_alg2_f64.argtypes = L.brsvd_run_alg2.argtypes
    L.brsvd_philox_normal_f64.argtypes = L.brsvd_philox_normal.argtypes
    L.brsvd_probe.argtypes = [i32, vp, u64, C.POINTER(dbl), C.POINTER(dbl), vp]
    L.brsvd_gemm_plan.argtypes = [i32, i64, i64, i32, i64, i32, C.POINTER(i32)]
    L.brsvd_destroy.argtypes = [vp]
    L.brsvd_status_string.argtypes = [C.c_int]
    L.brsvd_status_string.restype = C.c_char_p
    L.brsvd_gemm_an.argtypes = [vp, i64, i64, i64, vp, i32, vp, vp, u64, vp]
    L.brsvd_gemm_at.argtypes = [vp, i64, i64, i64, vp, i32, vp, i32, vp, u64, vp]
    L.brsvd_gemm_scratch_bytes.argtypes = [i64, i64, i32]
    L.brsvd_gemm_an_f64.argtypes = L.brsvd_gemm_an.argtypes
    L.brsvd_gemm_at_f64.argtypes = L.brsvd_gemm_at.argtypes
    L.brsvd_gemm_scratch_bytes_f64.argtypes = [i64, i64, i32]
    L.brsvd_orth.argtypes = [vp, i64, i32, i32, vp, C.POINTER(i32), vp, u64, vp]
    L.brsvd_orth_scratch_bytes.argtypes = [i64, i32]
    L.brsvd_small_svd.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32), vp, u64, vp]
    L.brsvd_small_svd_scratch_bytes.argtypes = [i32]
    L.brsvd_small_svd_static.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32), vp]
    sizes = ("brsvd_gemm_scratch_bytes", "brsvd_gemm_scratch_bytes_f64", "brsvd_orth_scratch_bytes",
             "brsvd_small_svd_scratch_bytes")
    for name in EXPORTS + STEP_EXPORTS:
        if name in sizes:
            getattr(L, name).restype = u64
        elif name != "brsvd_status_string":
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def brsvd_status_string(status: int) -> str:
    return lib().brsvd_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != BRSVD_OK:
        raise BrsvdError(status, where)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dev(t, dtype, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous CUDA tensor of dtype {dtype}")
    return t.data_ptr()


def make_params(m, n, k, p, q, row_block=0, device_budget_bytes=0, a_location=BRSVD_A_DEVICE,
                orth_method=BRSVD_ORTH_AUTO, compute_stream=None, copy_stream=None,
                pass_mode=BRSVD_PASSES_SEPARATE, dtype=BRSVD_DTYPE_F32, timing_level=0,
                workspace=None) -> brsvd_params:
    """workspace: optional CUDA uint8 tensor the handle uses instead of allocating (keep it alive)."""
    return brsvd_params(workspace=workspace.data_ptr() if workspace is not None else None,
                        workspace_bytes=workspace.numel() * workspace.element_size() if workspace is not None else 0,
                        m=m, n=n, k=k, p=p, q=q, a_location=a_location, row_block=row_block,
                        device_budget_bytes=device_budget_bytes, orth_method=orth_method, pass_mode=pass_mode,
                        compute_stream=_stream_ptr(compute_stream),
                        copy_stream=_stream_ptr(copy_stream) if copy_stream is not None else None,
                        dtype=dtype, timing_level=timing_level)


def brsvd_workspace_bytes(params: brsvd_params) -> int:
    out = C.c_uint64(0)
    _check(lib().brsvd_workspace_bytes(C.byref(params), C.byref(out)), "brsvd_workspace_bytes")
    return out.value


def brsvd_create(params: brsvd_params) -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().brsvd_create(C.byref(params), C.byref(h)), "brsvd_create")
    return h


def brsvd_destroy(handle) -> None:
    _check(lib().brsvd_destroy(handle), "brsvd_destroy")


def brsvd_run(handle, A, Omega, U=None, S=None, Vt=None, lda: Optional[int] = None, want_stats=True,
              pinned=False):
    """A: (m, n) CUDA tensor (or pinned host tensor for a host-resident handle), row stride lda, fp32 -- or
    fp64 for a handle created with dtype=BRSVD_DTYPE_F64 (brsvd_run_f64); Omega: (n, l) CUDA, same dtype.
    pinned=True vouches for a host A that torch did not allocate itself (see PinnedMatrix).
    Returns (U, S, Vt, stats) as CUDA tensors m x l, l, l x n."""
    import torch
    m, n = A.shape
    l = Omega.shape[1]
    dt = A.dtype
    if dt not in (torch.float32, torch.float64) or A.stride(1) != 1:
        raise TypeError("A must be fp32 or fp64 with unit column stride")
    if not A.is_cuda and not (pinned or A.is_pinned()):
        raise TypeError("a host-resident A must be pinned")
    lda = lda if lda is not None else A.stride(0)
    dev = Omega.device
    U = torch.empty(m, l, device=dev, dtype=dt) if U is None else U
    S = torch.empty(l, device=dev, dtype=dt) if S is None else S
    Vt = torch.empty(l, n, device=dev, dtype=dt) if Vt is None else Vt
    st = brsvd_stats()
    fn = lib().brsvd_run_f64 if dt == torch.float64 else lib().brsvd_run
    status = fn(handle, A.data_ptr(), lda, _dev(Omega, dt, "Omega"), _dev(U, dt, "U"), _dev(S, dt, "S"),
                _dev(Vt, dt, "Vt"), C.byref(st) if want_stats else None)
    _check(status, "brsvd_run")
    return U, S, Vt, (st.as_dict() if want_stats else None)


def brsvd_run_alg2(handle, A, l, seed=0, Omega=None, lda: Optional[int] = None, want_stats=True, pinned=False,
                   device=None):
    """Block-local scheme of Alg. 2.  A as for brsvd_run (fp32, or fp64 on a BRSVD_DTYPE_F64 handle); Omega
    (m, l) CUDA of the same dtype or None (then the library draws it from `seed`).  Returns (U, S, Vt, stats)."""
    import torch
    m, n = A.shape
    dt = A.dtype
    if dt not in (torch.float32, torch.float64) or A.stride(1) != 1:
        raise TypeError("A must be fp32 or fp64 with unit column stride")
    if not A.is_cuda and not (pinned or A.is_pinned()):
        raise TypeError("a host-resident A must be pinned")
    lda = lda if lda is not None else A.stride(0)
    dev = device or (Omega.device if Omega is not None else (A.device if A.is_cuda else torch.device("cuda:0")))
    U = torch.empty(m, l, device=dev, dtype=dt)
    S = torch.empty(l, device=dev, dtype=dt)
    Vt = torch.empty(l, n, device=dev, dtype=dt)
    st = brsvd_stats()
    fn = lib().brsvd_run_alg2_f64 if dt == torch.float64 else lib().brsvd_run_alg2
    status = fn(handle, A.data_ptr(), lda, int(seed), _dev(Omega, dt, "Omega") if Omega is not None else None,
                U.data_ptr(), S.data_ptr(), Vt.data_ptr(), C.byref(st) if want_stats else None)
    _check(status, "brsvd_run_alg2")
    return U, S, Vt, (st.as_dict() if want_stats else None)


def brsvd_gemm_plan(which, rows, n, l, block_rows=0, dtype=BRSVD_DTYPE_F32):
    """The launch plan of gemm_an (which = 0) or gemm_at (which = 1) as a list of 12 ints (see brsvd.h)."""
    out = (C.c_int32 * 12)()
    _check(lib().brsvd_gemm_plan(which, rows, n, l, block_rows, dtype, out), "brsvd_gemm_plan")
    return list(out)


def brsvd_probe(kind, buf, amount):
    """Measured device peaks: kind 0 streaming read of `amount` bytes of buf, kind 1 an fp32 MFMA loop.
    Returns (seconds, work) with work in bytes or flops."""
    sec, work = C.c_double(0.0), C.c_double(0.0)
    _check(lib().brsvd_probe(kind, buf.data_ptr(), int(amount), C.byref(sec), C.byref(work), None), "brsvd_probe")
    return sec.value, work.value


def brsvd_philox_normal(seed, rows, cols, row0=0, device="cuda:0", stream=None, f64=False):
    """Rows [row0, row0 + rows) of the Gaussian matrix brsvd_run_alg2 draws from `seed` (fp32, or fp64)."""
    import torch
    out = torch.empty(rows, cols, device=device, dtype=torch.float64 if f64 else torch.float32)
    fn = lib().brsvd_philox_normal_f64 if f64 else lib().brsvd_philox_normal
    _check(fn(int(seed), row0, rows, cols, out.data_ptr(), _stream_ptr(stream)), "brsvd_philox_normal")
    return out


def brsvd_rpca_ialm(handle, M, Omegas, iters, lam, mu0, rho, norm2_M=0.0, L=None, S=None, work=None):
    import torch
    m, n = M.shape
    L = torch.empty_like(M) if L is None else L
    S = torch.empty_like(M) if S is None else S
    work = torch.empty(2 * m * n, device=M.device) if work is None else work
    res = (C.c_double * iters)()
    st = brsvd_stats()
    status = lib().brsvd_rpca_ialm(handle, _dev(M, torch.float32, "M"), _dev(Omegas, torch.float32, "Omegas"),
                                   iters, lam, mu0, rho, norm2_M, _dev(L, torch.float32, "L"),
                                   _dev(S, torch.float32, "S"), _dev(work, torch.float32, "work"), res,
                                   C.byref(st))
    _check(status, "brsvd_rpca_ialm")
    return L, S, list(res), st.as_dict()


def brsvd_rpca_ialm_tol(handle, M, Omegas, max_iters, tol, lam, mu0, rho, norm2_M=0.0, L=None, S=None, work=None):
    """Returns L, S, the residuals of the iterations run, their number, and the statistics.  fp32, or fp64 when M
    is a float64 tensor (handle created with dtype=BRSVD_DTYPE_F64)."""
    import torch
    m, n = M.shape
    dt = M.dtype
    L = torch.empty_like(M) if L is None else L
    S = torch.empty_like(M) if S is None else S
    work = torch.empty(2 * m * n, device=M.device, dtype=dt) if work is None else work
    res = (C.c_double * max_iters)()
    done = C.c_int32(0)
    st = brsvd_stats()
    fn = lib().brsvd_rpca_ialm_tol_f64 if dt == torch.float64 else lib().brsvd_rpca_ialm_tol
    status = fn(handle, _dev(M, dt, "M"), _dev(Omegas, dt, "Omegas"), max_iters, tol, lam, mu0, rho, norm2_M,
                _dev(L, dt, "L"), _dev(S, dt, "S"), _dev(work, dt, "work"), res, C.byref(done), C.byref(st))
    _check(status, "brsvd_rpca_ialm_tol")
    return L, S, list(res)[:done.value], done.value, st.as_dict()


def brsvd_norm2_power(handle, A, x0, iters, lda=None) -> float:
    import torch
    out = C.c_double(0.0)
    lda = A.stride(0) if lda is None else lda
    fn = lib().brsvd_norm2_power_f64 if A.dtype == torch.float64 else lib().brsvd_norm2_power
    _check(fn(handle, A.data_ptr(), lda, _dev(x0, A.dtype, "x0"), iters, C.byref(out)), "brsvd_norm2_power")
    return out.value


def brsvd_gemm_scratch_bytes(rows, n, l, f64=False) -> int:
    L = lib()
    return (L.brsvd_gemm_scratch_bytes_f64 if f64 else L.brsvd_gemm_scratch_bytes)(rows, n, l)


def _scratch(rows, n, l, device, f64=False):
    import torch
    nbytes = brsvd_gemm_scratch_bytes(rows, n, l, f64)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device), nbytes


def brsvd_gemm_an(A, X, Y=None, rows=None, lda=None, stream=None):
    """Y = A[:rows] @ X on the HIP path.  A (rows, n) CUDA (row stride lda), X (n, l); fp32, or fp64 when
    A is a float64 tensor (brsvd_gemm_an_f64)."""
    import torch
    rows = A.shape[0] if rows is None else rows
    n = A.shape[1]
    l = X.shape[1]
    f64 = A.dtype == torch.float64
    dt = A.dtype
    lda = A.stride(0) if lda is None else lda
    Y = torch.empty(rows, l, device=X.device, dtype=dt) if Y is None else Y
    scr, nbytes = _scratch(rows, n, l, X.device, f64)
    fn = lib().brsvd_gemm_an_f64 if f64 else lib().brsvd_gemm_an
    _check(fn(A.data_ptr(), lda, rows, n, _dev(X, dt, "X"), l, _dev(Y, dt, "Y"), scr.data_ptr(), nbytes,
              _stream_ptr(stream)), "brsvd_gemm_an")
    return Y


def brsvd_gemm_at(A, Q, Z=None, accumulate=False, lda=None, stream=None):
    """Z (+)= A^T @ Q on the HIP path.  A (rows, n), Q (rows, l), Z (n, l); fp32 or fp64 by A's dtype."""
    import torch
    rows, n = A.shape
    l = Q.shape[1]
    f64 = A.dtype == torch.float64
    dt = A.dtype
    lda = A.stride(0) if lda is None else lda
    Z = torch.zeros(n, l, device=Q.device, dtype=dt) if Z is None else Z
    scr, nbytes = _scratch(rows, n, l, Q.device, f64)
    fn = lib().brsvd_gemm_at_f64 if f64 else lib().brsvd_gemm_at
    _check(fn(A.data_ptr(), lda, rows, n, _dev(Q, dt, "Q"), l, _dev(Z, dt, "Z"), 1 if accumulate else 0,
              scr.data_ptr(), nbytes, _stream_ptr(stream)), "brsvd_gemm_at")
    return Z


def _byte_scratch(nbytes, device):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def brsvd_orth(P, method=BRSVD_ORTH_AUTO, want_R=False, stream=None):
    """In-place orthonormalisation of the columns of P (rows, l).  Returns (P, R or None, fallback)."""
    import torch
    rows, l = P.shape
    R = torch.empty(l, l, dtype=torch.float64, device=P.device) if want_R else None
    fb = C.c_int32(0)
    nbytes = lib().brsvd_orth_scratch_bytes(rows, l)
    scr = _byte_scratch(nbytes, P.device)
    _check(lib().brsvd_orth(_dev(P, torch.float32, "P"), rows, l, method, R.data_ptr() if want_R else None,
                            C.byref(fb), scr.data_ptr(), nbytes, _stream_ptr(stream)), "brsvd_orth")
    return P, R, bool(fb.value)


def brsvd_small_svd(R, stream=None, out=None, static=False):
    """One-sided Jacobi SVD of an l x l fp64 CUDA matrix: returns (S, Ur, Vr, sweeps).  out = (S, Ur, Vr)
    reuses the caller's tensors; static=True calls brsvd_small_svd_static (scratch inside the library)."""
    import torch
    l = R.shape[0]
    if out is None:
        out = (torch.empty(l, dtype=torch.float64, device=R.device),
               torch.empty(l, l, dtype=torch.float64, device=R.device),
               torch.empty(l, l, dtype=torch.float64, device=R.device))
    S, Ur, Vr = out
    sw = C.c_int32(0)
    args = (_dev(R, torch.float64, "R"), l, _dev(S, torch.float64, "S"), _dev(Ur, torch.float64, "Ur"),
            _dev(Vr, torch.float64, "Vr"), C.byref(sw))
    if static:
        _check(lib().brsvd_small_svd_static(*args, _stream_ptr(stream)), "brsvd_small_svd_static")
    else:
        nbytes = lib().brsvd_small_svd_scratch_bytes(l)
        scr = _byte_scratch(nbytes, R.device)
        _check(lib().brsvd_small_svd(*args, scr.data_ptr(), nbytes, _stream_ptr(stream)), "brsvd_small_svd")
    return S, Ur, Vr, sw.value


def brsvd_small_svd_static(R, stream=None, out=None):
    return brsvd_small_svd(R, stream=stream, out=out, static=True)


class PinnedMatrix:
    """rows x cols fp32 matrix in pinned host memory obtained with one hipHostMalloc of the exact size
    (torch's pinned allocator rounds requests up to a power of two, which fails for very large A).
    `.tensor` is a torch view of the memory; call `.free()` when done."""

    def __init__(self, rows: int, cols: int):
        import numpy as np
        import torch
        self._hip = C.CDLL("libamdhip64.so")
        self._hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
        self._hip.hipHostFree.argtypes = [C.c_void_p]
        ptr = C.c_void_p()
        err = self._hip.hipHostMalloc(C.byref(ptr), rows * cols * 4, 0)
        if err != 0 or not ptr.value:
            self._hip.hipGetLastError()          # the failure is reported here; do not leave it for the next HIP call
            raise MemoryError(f"hipHostMalloc of {rows * cols * 4} bytes failed (hip error {err})")
        self.ptr = ptr.value
        buf = (C.c_float * (rows * cols)).from_address(self.ptr)
        self.tensor = torch.from_numpy(np.ctypeslib.as_array(buf)).view(rows, cols)

    def free(self):
        if self.ptr:
            self.tensor = None
            self._hip.hipHostFree(C.c_void_p(self.ptr))
            self.ptr = None
