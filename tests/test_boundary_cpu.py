"""Host-side checks that need no GPU: the shared library loads, exports every symbol declared in
include/brsvd.h, validates its arguments and sizes its working set."""
import ctypes as C
import os
import re

import pytest

import paper_1706_07191_amd as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    for header, exports in (("brsvd.h", B.EXPORTS), ("brsvd_steps.h", B.STEP_EXPORTS)):
        hdr = open(os.path.join(ROOT, "include", header)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)          # declarations only, not the comments
        declared = set(re.findall(r"\b(brsvd_[a-z_0-9]+)\s*\(", hdr))
        assert declared == set(exports), header
        for name in declared:
            assert getattr(L, name) is not None
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["brsvd.h", "brsvd_steps.h"]


def test_product_path_does_not_import_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_1706_07191_amd")):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in txt and "from oracle" not in txt, f


def test_status_strings():
    assert B.brsvd_status_string(0) == "ok"
    for s in range(-6, 0):
        assert B.brsvd_status_string(s) not in ("ok", "unknown status")
    assert B.brsvd_status_string(-99) == "unknown status"


def _p(**kw):
    base = dict(m=2000, n=1000, k=20, p=10, q=2, row_block=512)
    base.update(kw)
    return B.brsvd_params(a_location=kw.pop("a_location", 0), pass_mode=base.pop("pass_mode", 0), orth_method=0,
                          device_budget_bytes=base.pop("device_budget_bytes", 0),
                          compute_stream=None, copy_stream=None, **{k: v for k, v in base.items()
                                                                    if k not in ("a_location",)})


@pytest.mark.parametrize("bad", [dict(m=0), dict(n=-1), dict(k=0), dict(p=-1), dict(q=-1),
                                 dict(k=600, p=0), dict(m=20, n=1000), dict(row_block=-5), dict(pass_mode=7), dict(dtype=5),
                                 dict(timing_level=3)])
def test_invalid_params_rejected(bad):
    out = C.c_uint64(0)
    assert B.lib().brsvd_workspace_bytes(C.byref(_p(**bad)), C.byref(out)) == B.BRSVD_ERR_ARG
    h = C.c_void_p()
    assert B.lib().brsvd_create(C.byref(_p(**bad)), C.byref(h)) == B.BRSVD_ERR_ARG
    assert not h


def test_null_arguments_rejected():
    L = B.lib()
    assert L.brsvd_workspace_bytes(None, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_create(None, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_run(None, None, 0, None, None, None, None, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_destroy(None) == B.BRSVD_OK
    assert L.brsvd_gemm_an(None, 0, 0, 0, None, 0, None, None, 0, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_gemm_at(None, 0, 0, 0, None, 0, None, 0, None, 0, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_orth(None, 0, 0, 0, None, None, None, 0, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_small_svd(None, 0, None, None, None, None, None, 0, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_small_svd_static(None, 0, None, None, None, None, None) == B.BRSVD_ERR_ARG
    # sizes beyond the scratch the no-allocation call carries, and scratch that is missing, misaligned or short:
    # all rejected on the host, before any GPU call
    one = C.c_void_p(256)
    assert L.brsvd_small_svd_static(one, 513, one, one, one, None, None) == B.BRSVD_ERR_BUDGET
    assert L.brsvd_small_svd(one, 8, one, one, one, None, None, 1 << 20, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_small_svd(one, 8, one, one, one, None, C.c_void_p(264), 1 << 20, None) == B.BRSVD_ERR_ARG
    assert L.brsvd_small_svd(one, 8, one, one, one, None, one, 16, None) == B.BRSVD_ERR_BUDGET
    assert L.brsvd_orth(one, 100, 8, 0, None, None, one, 16, None) == B.BRSVD_ERR_BUDGET
    assert L.brsvd_small_svd_scratch_bytes(8) >= 2 * 16 * 16 * 8 and L.brsvd_small_svd_scratch_bytes(0) == 0
    assert L.brsvd_orth_scratch_bytes(100, 8) >= 2 * 100 * 16 * 4 and L.brsvd_orth_scratch_bytes(100, 600) == 0


def test_workspace_accounting_and_budget():
    small = B.brsvd_workspace_bytes(_p())
    # at least the four thin panels (l = 30 padded to 32)
    assert small >= 2 * (2000 + 1000) * 32 * 4
    big = B.brsvd_workspace_bytes(_p(m=20000, n=20000, k=100, p=10, row_block=4096))
    assert big > small
    out = C.c_uint64(0)
    st = B.lib().brsvd_workspace_bytes(C.byref(_p(device_budget_bytes=small - 1)), C.byref(out))
    assert st == B.BRSVD_ERR_BUDGET
    assert B.brsvd_workspace_bytes(_p(device_budget_bytes=small)) == small
    # host-resident A adds the two staging blocks
    host = B.brsvd_workspace_bytes(_p(a_location=B.BRSVD_A_HOST_PINNED))
    assert host >= 2 * (2000 + 1000) * 32 * 4 + 2 * 512 * 1000 * 4
    assert B.brsvd_gemm_scratch_bytes(512, 1000, 30) > 0
    assert B.brsvd_gemm_scratch_bytes(0, 1000, 30) == 0
    # a caller's workspace bounds the working set exactly as the budget does; it must be 256-byte aligned
    h = C.c_void_p()
    p = _p()
    p.workspace, p.workspace_bytes = 4096, small - 1
    assert B.lib().brsvd_create(C.byref(p), C.byref(h)) == B.BRSVD_ERR_BUDGET and not h
    p.workspace, p.workspace_bytes = 4100, small
    assert B.lib().brsvd_create(C.byref(p), C.byref(h)) == B.BRSVD_ERR_ARG and not h
    # the split-sum scratch of A X covers the leftover row tiles only: C3's in-core working set stays near its
    # four panels (2 x 100000 x 272 + 2 x 50000 x 272 floats = 163 MB) instead of carrying 2 GB of scratch
    c3 = B.brsvd_workspace_bytes(_p(m=100000, n=50000, k=256, p=16, q=1, row_block=8192))
    assert c3 < 1.7e9        # of which about 1 GB are the partial panels of the split A^T Q launch
