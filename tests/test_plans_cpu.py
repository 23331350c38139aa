"""Host-side invariants of the launch plans of the two thin products (no GPU needed).

The decode below restates, in Python, how a workgroup of k_gemm_an derives its work from the plan
numbers; the test then checks that every (row tile, chunk) unit is covered exactly once, that partial
panels never exceed the scratch the library asks for, and that the sub-ranges of gemm_at tile every
row block."""
import random

import pytest

import paper_1706_07191_amd as B


def _an_segments(plan):
    tile_rows, T, C, whole, lt, f, x, j, nsplit, wgs, groups, nt = plan
    segs = []                                    # (workgroup, tile, c0, c1, slot or None for direct)
    for b in range(wgs):
        if b < whole:
            segs.append((b, b, 0, C, None))
        elif b < whole + lt * f:
            idx = b - whole
            s = idx % f
            segs.append((b, whole + idx // f, s * (C - x) // f, (s + 1) * (C - x) // f, s))
        else:
            i = b - whole - lt * f
            first = whole + i * j
            for t in range(first, min(first + j, whole + lt)):
                segs.append((b, t, C - x, C, f))
    return segs


def _check_an(rows, K, l, dtype):
    plan = B.brsvd_gemm_plan(0, rows, K, l, 0, dtype)
    tile_rows, T, C, whole, lt, f, x, j, nsplit, wgs, groups, nt = plan
    esz = 8 if dtype == B.BRSVD_DTYPE_F64 else 4
    Lp = (l + 15) // 16 * 16
    assert T == -(-rows // tile_rows) and whole + lt == T and groups * nt * 16 >= Lp
    narrow = esz == 4 and nt == 1 and K >= 512   # fp32 panels of one column tile over long rows: 32-row tiles, 256-column chunks
    kc = 256 if narrow else (32 if (esz == 8 or nt > 8) else 64)
    assert tile_rows == 32 if narrow else tile_rows % 16 == 0
    assert C == -(-K // kc)
    cover = {}
    last_wg = -1
    for wg, t, c0, c1, slot in _an_segments(plan):
        assert 0 <= t < T and 0 <= c0 < c1 <= C, (plan, wg, t, c0, c1)
        assert wg >= last_wg
        last_wg = wg
        if slot is None:
            assert t < whole
        else:
            assert t >= whole and 0 <= slot < nsplit
        cover.setdefault(t, []).append((c0, c1, slot))
    assert last_wg == wgs - 1 and set(cover) == set(range(T))
    for t, ranges in cover.items():
        ranges.sort()
        assert ranges[0][0] == 0 and ranges[-1][1] == C
        for (a0, a1, _), (b0, b1, _) in zip(ranges, ranges[1:]):
            assert a1 == b0                       # contiguous, no overlap
        slots = [s for _, _, s in ranges]
        assert slots == [None] or slots == list(range(len(slots))) and len(slots) == nsplit
    # scratch of the split sums: nsplit partial panels of the rows of the leftover tiles only (not of all rows)
    leftover_rows = rows - whole * tile_rows if nsplit else 0
    sizes = B.brsvd_gemm_plan(2, rows, K, l, 0, dtype)
    an_bytes = sizes[0] + (sizes[1] << 31)
    assert an_bytes == nsplit * leftover_rows * Lp * esz
    panel = -(-max(rows, K) * Lp * esz // 256) * 256
    assert B.brsvd_gemm_scratch_bytes(rows, K, l, f64=esz == 8) >= 2 * panel + an_bytes


@pytest.mark.parametrize("rows,K,l", [(20000, 20000, 110), (100000, 50000, 272), (76800, 2000, 20), (2073600, 100, 20),
                                      (1000, 1000, 30), (64, 8, 1), (9000, 2100, 64), (65536 + 128, 4096, 16),
                                      (700, 1536, 512), (129, 1025, 17), (128 * 512, 64 * 16, 32), (128 * 513, 64 * 17, 32)])
@pytest.mark.parametrize("dtype", [B.BRSVD_DTYPE_F32, B.BRSVD_DTYPE_F64])
def test_gemm_an_plan_covers_every_unit_once(rows, K, l, dtype):
    _check_an(rows, K, l, dtype)


def test_gemm_an_plan_random_shapes():
    rng = random.Random(1706)
    for _ in range(400):
        rows = rng.choice([rng.randint(1, 300), rng.randint(1, 70000), rng.randint(60000, 600000)])
        K = rng.choice([rng.randint(1, 200), rng.randint(1, 5000), rng.randint(1000, 120000)])
        l = rng.randint(1, 512)
        _check_an(rows, K, l, rng.choice([B.BRSVD_DTYPE_F32, B.BRSVD_DTYPE_F64]))


def test_gemm_at_plan_tiles_every_block():
    rng = random.Random(7191)
    shapes = [(20000, 20000, 110, 4096), (100000, 50000, 272, 8192), (2073600, 100, 20, 65536), (77, 1003, 20, 0),
              (16384, 100000, 144, 16384)]
    for _ in range(300):
        rows = rng.randint(1, 300000)
        shapes.append((rows, rng.randint(1, 60000), rng.randint(1, 512), rng.choice([0, rng.randint(1, rows)])))
    for rows, n, l, b in shapes:
        for dtype in (B.BRSVD_DTYPE_F32, B.BRSVD_DTYPE_F64):
            mt, waves, col_tiles, nblocks, sub, rps, nsplit, kc, groups, nt, _, _ = B.brsvd_gemm_plan(1, rows, n, l, b, dtype)
            block = rows if b <= 0 or b > rows else b
            assert nblocks == -(-rows // block) and nsplit == nblocks * sub
            assert col_tiles * waves * mt * 16 >= n > (col_tiles - 1) * waves * mt * 16
            assert rps % kc == 0 and sub * rps >= block and (sub - 1) * rps < block      # sub-ranges tile the block
            assert groups * nt * 16 >= (l + 15) // 16 * 16
