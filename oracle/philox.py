"""Counter-based Gaussian generator for the test matrices that Alg. 2 draws on the device.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Written from the published algorithm, not from
the HIP code: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as
easy as 1, 2, 3", SC'11) followed by the Box-Muller transform.  The HIP library implements the same
definition on its own, so that both sides can draw the same Omega from a seed.

Definition of the matrix Omega(seed; rows x cols), row-major, element e = row * cols + col:
    counter = (e >> 2) as a 128-bit little-endian number in four 32-bit words, key = (seed low word,
    seed high word); x0..x3 = Philox4x32-10(counter, key);
    u(x) = ((x >> 9) + 0.5) * 2^-23                       (23-bit uniform in (0, 1); with the half added it
                                                           still fits the 24-bit significand of fp32)
    z0 = sqrt(-2 ln u(x0)) cos(2 pi u(x1)),  z1 = sqrt(-2 ln u(x0)) sin(2 pi u(x1)),
    z2, z3 likewise from (x2, x3);  Omega[e] = z_(e & 3).
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key) -> np.ndarray:
    """counter: (..., 4) array of 32-bit words (any integer dtype), key: two 32-bit words.
    Returns the (..., 4) uint32 outputs of ten Philox rounds."""
    c = np.asarray(counter).astype(np.uint64) & _MASK
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for _ in range(10):
        p0 = _M0 * c0                      # 64-bit products of 32-bit operands
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + _W0) & _MASK
        k1 = (k1 + _W1) & _MASK
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def _uniform23(x: np.ndarray) -> np.ndarray:
    return ((x >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def philox_normal(seed: int, rows: int, cols: int, row0: int = 0) -> np.ndarray:
    """Rows [row0, row0 + rows) of Omega(seed; * x cols) as fp64 (see the module docstring)."""
    e0 = row0 * cols
    e1 = (row0 + rows) * cols
    c_first, c_last = e0 >> 2, (e1 + 3) >> 2
    idx = np.arange(c_first, c_last, dtype=np.uint64)
    ctr = np.zeros((idx.size, 4), dtype=np.uint64)
    ctr[:, 0] = idx & _MASK
    ctr[:, 1] = idx >> _S32
    x = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    r01 = np.sqrt(-2.0 * np.log(_uniform23(x[:, 0])))
    t01 = 2.0 * np.pi * _uniform23(x[:, 1])
    r23 = np.sqrt(-2.0 * np.log(_uniform23(x[:, 2])))
    t23 = 2.0 * np.pi * _uniform23(x[:, 3])
    z = np.stack([r01 * np.cos(t01), r01 * np.sin(t01), r23 * np.cos(t23), r23 * np.sin(t23)], axis=1).reshape(-1)
    off = e0 - 4 * c_first
    return z[off:off + rows * cols].reshape(rows, cols)
