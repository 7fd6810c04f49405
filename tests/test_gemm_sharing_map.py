"""The index arithmetic of the GEMM's shared last round (which block takes which K tiles of which
tile, where its partial tile goes, which partial tiles the fix-up kernel adds for a tile), checked on
the CPU by brute force through the library's host-side test aids.  No device work."""
import ctypes
import os

import numpy as np
import pytest


@pytest.fixture(scope="module")
def libqii():
    from paper_2601_22813_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=True)
    return binding


def _segments(L, rem, ktotal, grid):
    out = (ctypes.c_int32 * 20)()
    segs = []
    for block_id in range(grid):
        n = L.qii_gemm_sharing_segments(rem, ktotal, grid, block_id, out)
        assert n >= 1, (rem, ktotal, grid, block_id, n)
        segs += [tuple(out[5 * i:5 * i + 5]) for i in range(n)]
    return segs


def _check(L, rem, ktotal, grid):
    segs = _segments(L, rem, ktotal, grid)
    # block numbers are a permutation of the hardware block ids
    assert sorted({s[0] for s in segs}) == list(range(grid))
    # every K tile of every shared tile is taken exactly once
    cover = np.zeros((rem, ktotal), np.int32)
    for blk, lt, kt0, kts, slot in segs:
        assert 0 <= lt < rem and 0 <= kt0 and kts >= 1 and kt0 + kts <= ktotal
        cover[lt, kt0:kt0 + kts] += 1
    assert (cover == 1).all()
    # partial-tile slots: unique, inside the workspace area of grid + rem tiles
    slots = [s[4] for s in segs]
    assert len(set(slots)) == len(slots) and min(slots) >= 0 and max(slots) < grid + rem
    # equal ranges: block sizes differ by at most one unit; at most two segments per block when a
    # range is no longer than a tile's K
    per_block = {}
    for blk, lt, kt0, kts, slot in segs:
        per_block.setdefault(blk, []).append(kts)
    sizes = [sum(v) for v in per_block.values()]
    assert max(sizes) - min(sizes) <= 1
    if max(sizes) <= ktotal:
        assert max(len(v) for v in per_block.values()) <= 2
    # the slots the fix-up kernel adds up for a tile are exactly that tile's segments, consecutive
    # and in the order of their K ranges
    by_slot = {s[4]: s for s in segs}
    out2 = (ctypes.c_int32 * 2)()
    for lt in range(rem):
        L.qii_gemm_sharing_tile_slots(rem, ktotal, grid, lt, out2)
        first, last = out2[0], out2[1]
        k = 0
        for slot in range(first, last + 1):
            blk, t, kt0, kts, _ = by_slot[slot]
            assert t == lt and kt0 == k
            k += kts
        assert k == ktotal
        assert sum(1 for s in segs if s[1] == lt) == last - first + 1


def test_sharing_map_small_and_ragged_cases(libqii):
    L = libqii.lib()
    L.qii_gemm_sharing_segments.restype = ctypes.c_int
    for rem, ktotal, grid in [(1, 8, 2), (1, 16, 4), (4, 32, 32), (6, 16, 24), (5, 24, 24), (8, 16, 32), (64, 128, 256),
                              (96, 64, 256), (144, 64, 256), (255, 8, 256), (7, 9, 8), (3, 100, 72), (13, 37, 120)]:
        _check(L, rem, ktotal, grid)


def test_sharing_map_random_cases_follow_the_plan_rule(libqii):
    """grid as the plan chooses it: min(256, units / 4), a multiple of 8 from 8 on, more blocks than tiles."""
    L = libqii.lib()
    L.qii_gemm_sharing_segments.restype = ctypes.c_int
    rng = np.random.default_rng(5)
    done = 0
    while done < 60:
        rem, ktotal = int(rng.integers(1, 256)), int(rng.integers(8, 200))
        grid = min(256, rem * ktotal // 4)
        if grid >= 8:
            grid &= ~7
        if grid <= rem:
            continue
        _check(L, rem, ktotal, grid)
        done += 1


@pytest.mark.parametrize("M,N,K,expect", [
    (16384, 8192, 2048, (2048, 0, 0)),       # whole rounds
    (2048, 2048, 32768, (0, 64, 256)),        # fewer tiles than compute units, long K
    (11264, 2048, 16384, (256, 96, 256)),     # one full round, 96 shared tiles
    (2048, 5632, 16384, (176, 0, 0)),         # 176 tiles: sharing would not pay
    (512, 512, 8192, (0, 4, 32)),             # 4 tiles, 128 units: 32 blocks of 4
    (300, 200, 384, (2, 0, 0)),               # K not a multiple of 256: another kernel, no plan
])
def test_sharing_plan_of_known_shapes(libqii, M, N, K, expect):
    L = libqii.lib()
    plan = (ctypes.c_int32 * 3)()
    L.qii_gemm_sharing_plan(ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), plan)
    assert tuple(plan) == expect
    # the workspace has room for one partial tile per sharing block and shared tile behind the scale bytes
    up = lambda r: (r + 255) // 256 * 256
    scales = (up(M) + up(N)) * (K // 16) if K % 256 == 0 else 0
    extra = (plan[2] + plan[1]) * 256 * 256 * 4 if plan[1] else 0
    need = libqii.qii_gemm_workspace_bytes(M, N, K)
    assert scales + extra <= need <= scales + extra + 512
