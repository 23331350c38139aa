"""Builds libbrsvd.so (hand-written HIP for gfx950) in-tree with hipcc.

Usage: python -m paper_1706_07191_amd.build [--force]
       python -m paper_1706_07191_amd.build --host-asan
The shared library is written next to this file; object files go to csrc/_build/.
--host-asan builds csrc/_build_asan/host_checks instead: the same sources with their HOST code instrumented by
the address and undefined-behaviour sanitizers (the device code is compiled as usual and never runs), linked
with csrc/host_checks.cpp, which exercises argument checks, working-set sizing, the launch planners and the
failure paths of the runtime calls without needing a GPU.  Run the executable: exit status 0 = clean.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libbrsvd.so")
SOURCES = ["gemm_thin.hip", "orth.hip", "tsqr.hip", "small_svd.hip", "rpca.hip", "philox.hip", "probe.hip", "brsvd.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in r.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    headers = [os.path.join(CSRC, "common.h"), os.path.join(ROOT, "include", "brsvd.h"),
               os.path.join(ROOT, "include", "brsvd_steps.h")]
    jobs = []
    objs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + headers):
            jobs.append([hipcc] + FLAGS + ["-c", s, "-o", o])
    with ThreadPoolExecutor(max_workers=min(6, max(1, len(jobs)))) as ex:
        for out in ex.map(_run, jobs):
            if verbose and out.strip():
                print(out)
    if force or jobs or _stale(LIB, objs):
        out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
        if verbose and out.strip():
            print(out)
    return LIB


ASAN_DIR = os.path.join(CSRC, "_build_asan")
ASAN_EXE = os.path.join(ASAN_DIR, "host_checks")
# each -fsanitize goes directly behind -Xarch_host: only the host pass is instrumented
ASAN_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
              "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_host_asan(force: bool = False, verbose: bool = False) -> str:
    """Builds csrc/_build_asan/host_checks (see the module docstring) and returns its path."""
    os.makedirs(ASAN_DIR, exist_ok=True)
    hipcc = _hipcc()
    headers = [os.path.join(CSRC, "common.h"), os.path.join(ROOT, "include", "brsvd.h"),
               os.path.join(ROOT, "include", "brsvd_steps.h")]
    base = [f for f in FLAGS if f != "-O3"]
    jobs, objs = [], []
    for src in SOURCES + ["host_checks.cpp"]:
        s = os.path.join(CSRC, src)
        o = os.path.join(ASAN_DIR, os.path.splitext(src)[0] + ".o")
        objs.append(o)
        if force or _stale(o, [s] + headers):
            lang = ["-x", "hip"] if src.endswith(".cpp") else []
            jobs.append([hipcc] + base + ASAN_FLAGS + lang + ["-c", s, "-o", o])
    with ThreadPoolExecutor(max_workers=min(6, max(1, len(jobs)))) as ex:
        for out in ex.map(_run, jobs):
            if verbose and out.strip():
                print(out)
    if force or jobs or _stale(ASAN_EXE, objs):
        out = _run([hipcc, "--offload-arch=gfx950", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                    "-fsanitize=undefined", "-o", ASAN_EXE] + objs)
        if verbose and out.strip():
            print(out)
    return ASAN_EXE


if __name__ == "__main__":
    if "--host-asan" in sys.argv:
        print(build_host_asan(force="--force" in sys.argv, verbose=True))
    else:
        print(build(force="--force" in sys.argv, verbose=True))
