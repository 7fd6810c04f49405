"""Pins of the oracle's number formats and generator against things other than itself:
the format definitions of Sec. 3.1 of the paper, a library cast (torch float8_e4m3fn),
brute force over the whole grid, and the published Philox known answers."""
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _constants():
    out = {}
    for line in open(os.path.join(GOLDEN, "format_constants.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


E2M1_MAGS = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_e2m1_decode_is_the_e2m1_format(oracle):
    # 1 sign, 2 exponent (bias 1), 1 mantissa bit, written out from the bit fields
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        v = (m * 0.5) if e == 0 else (1 + 0.5 * m) * 2.0 ** (e - 1)
        assert oracle.e2m1_decode(code) == (-v if s else v)
    assert max(oracle.e2m1_decode(c) for c in range(16)) == _constants()["fp4_max"]
    assert sorted({abs(oracle.e2m1_decode(c)) for c in range(16)}) == E2M1_MAGS


def test_e2m1_rtn_roundtrip_midpoints_saturation(oracle):
    for code in range(16):
        assert oracle.e2m1_rtn(oracle.e2m1_decode(code)) == code
    # the seven midpoints go to the neighbour with the even code
    for mid, want in [(0.25, 0.0), (0.75, 1.0), (1.25, 1.0), (1.75, 2.0), (2.5, 2.0), (3.5, 4.0),
                      (5.0, 4.0)]:
        assert oracle.e2m1_decode(oracle.e2m1_rtn(mid)) == want
        assert oracle.e2m1_decode(oracle.e2m1_rtn(-mid)) == -want
    for big in (6.0, 6.5, 100.0, 3e38):
        assert oracle.e2m1_decode(oracle.e2m1_rtn(big)) == 6.0
        assert oracle.e2m1_decode(oracle.e2m1_rtn(-big)) == -6.0
    assert oracle.e2m1_rtn(-0.1) == 8  # sign kept on a value that rounds to zero


def test_e2m1_rtn_is_nearest_by_brute_force(oracle):
    rng = np.random.default_rng(1)
    qs = np.concatenate([rng.uniform(-7, 7, 4000), rng.normal(0, 1, 2000),
                         np.nextafter(np.float32([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]), 10),
                         np.nextafter(np.float32([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]), -10)]
                        ).astype(np.float32)
    grid = np.array(E2M1_MAGS)
    for q in qs:
        got = abs(oracle.e2m1_decode(oracle.e2m1_rtn(float(q))))
        dist = np.abs(grid - abs(float(q)))
        assert abs(got - abs(float(q))) == dist.min()


def test_e4m3_decode_matches_torch_cast(oracle):
    bytes_ = torch.arange(0, 127, dtype=torch.uint8)
    want = bytes_.view(torch.float8_e4m3fn).float().numpy()
    got = np.array([oracle.e4m3_decode(int(b)) for b in range(127)], dtype=np.float32)
    assert np.array_equal(got, want)
    c = _constants()
    assert got.max() == c["fp8_max"]
    normals = got[8:]  # bytes 0x08.. are normal numbers
    ratios = normals[1:] / normals[:-1]
    # neighbours are at least a factor 1.0625 apart (the paper's bound; the tightest pair is
    # 1.875 -> 2, a factor 16/15) and at most 1.125
    assert ratios.min() >= c["fp8_min_relative_step"]
    assert ratios.min() == np.float32(16.0 / 15.0) and ratios.max() == 1.125
    assert np.all(np.diff(got) > 0)


def test_e4m3_rtn_shrinks_by_at_most_16_over_17(oracle):
    # Sec. 3.1: 16/17 is the largest factor by which RTN_FP8 can shrink a value (so dividing by
    # the rounded scale grows the normalized values by at most 17/16)
    c = _constants()
    assert c["rtn_fp8_margin"] == pytest.approx(16.0 / 17.0)
    rng = np.random.default_rng(5)
    worst = 1.0
    for r in np.exp(rng.uniform(np.log(2.0 ** -6), np.log(448.0), 20000)).astype(np.float32):
        worst = min(worst, oracle.e4m3_decode(oracle.e4m3_rtn(float(r))) / float(r))
    assert worst >= 16.0 / 17.0
    just_below_tie = float(np.nextafter(np.float32(1.0625), np.float32(0)))
    assert oracle.e4m3_decode(oracle.e4m3_rtn(just_below_tie)) == 1.0
    assert oracle.e4m3_decode(oracle.e4m3_rtn(just_below_tie)) / just_below_tie == pytest.approx(16 / 17, rel=1e-6)


def test_e4m3_rtn_matches_torch_cast_on_a_dense_sweep(oracle):
    rng = np.random.default_rng(2)
    vals = np.concatenate([
        np.exp(rng.uniform(np.log(1e-4), np.log(463.9), 20000)),
        rng.uniform(0, 2.0 ** -5, 3000),                     # subnormal range and around it
        np.array([oracle.e4m3_decode(b) for b in range(127)]),
        # exact midpoints between neighbours: ties must go to the even byte
        np.array([(oracle.e4m3_decode(b) + oracle.e4m3_decode(b + 1)) / 2 for b in range(126)]),
    ]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_rtn(float(v)) for v in vals], dtype=np.uint8)
    assert np.array_equal(got, want)
    # saturation at 448 and never the NaN byte
    for big in (448.0, 463.9, 464.0, 480.0, 1e6, 3e38):
        assert oracle.e4m3_rtn(big) == 0x7E
    assert oracle.e4m3_rtn(0.0) == 0 and oracle.e4m3_rtn(2.0 ** -11) == 0
    for b in range(127):
        assert oracle.e4m3_rtn(oracle.e4m3_decode(b)) == b


def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_draws_are_the_documented_words_of_philox(oracle):
    seed = 0x0123456789ABCDEF
    key = [seed & 0xFFFFFFFF, seed >> 32]
    # scale draw: counter (column group, row div 4, 0, stream), word row mod 4, top 20 bits
    for row, cg in [(0, 0), (5, 3), (1023, 511), (7, 0)]:
        w = oracle.philox4x32_10([cg, row >> 2, 0, 0x53434C00], key)
        assert oracle.scale_draw(seed, row, cg) == int(w[row & 3]) >> 12
    # element draw: counter (col div 8, row, 0, stream), 16-bit halves, low half first
    for row, col in [(0, 0), (0, 1), (3, 14), (100, 8191)]:
        w = oracle.philox4x32_10([col >> 3, row, 0, 0x454C4D00], key)
        word = int(w[(col & 7) >> 1])
        assert oracle.elem_draw(seed, row, col) == ((word >> 16) if col & 1 else (word & 0xFFFF))
    w = oracle.philox4x32_10([4, 0, 0, 0x44525600], key)
    assert oracle.derive_seed(seed, 4) == (int(w[1]) << 32) | int(w[0])
    signs = oracle.rht_signs(seed)
    w = oracle.philox4x32_10([0, 0, 0, 0x52485400], key)
    for j in range(128):
        assert signs[j] == (-1.0 if (int(w[j >> 5]) >> (j & 31)) & 1 else 1.0)
    assert 30 < (signs < 0).sum() < 98


def test_draws_look_uniform(oracle):
    # 2^14 scale draws: mean of R/2^20 is 1/2 within 5 sigma, all 4 words differ between rows
    draws = np.array([oracle.scale_draw(7, r, c) for r in range(128) for c in range(128)])
    u = draws / 2.0 ** 20
    assert abs(u.mean() - 0.5) < 5 * (1 / np.sqrt(12)) / np.sqrt(u.size)
    assert draws.max() < 2 ** 20 and len(np.unique(draws)) > 0.98 * draws.size
    e = np.array([oracle.elem_draw(7, r, c) for r in range(64) for c in range(256)]) / 65536.0
    assert abs(e.mean() - 0.5) < 5 * (1 / np.sqrt(12)) / np.sqrt(e.size)


def test_e2m1_sr_expectation_by_enumeration(oracle):
    # SR_FP4 preserves its argument in expectation (Sec. 3.1): enumerate all 2^16 draws
    for q in [0.1, 0.3, 0.74, 1.2, 1.9, 2.3, 3.99, 4.5, 5.9, -2.7, -0.01]:
        q32 = float(np.float32(q))
        vals = np.array([oracle.e2m1_decode(c) for c in range(16)])
        counts = np.zeros(16)
        # the draw only matters through a threshold, so count by bisection instead of 65536 calls
        lo_code = oracle.e2m1_sr(q32, 0)
        hi_code = oracle.e2m1_sr(q32, 65535)
        a, b = 0, 65535
        if lo_code == hi_code:
            counts[lo_code] = 65536
        else:
            while b - a > 1:
                mid = (a + b) // 2
                if oracle.e2m1_sr(q32, mid) == lo_code:
                    a = mid
                else:
                    b = mid
            counts[lo_code] = b
            counts[hi_code] = 65536 - b
            # monotone in the draw: spot-check both sides of the threshold
            assert oracle.e2m1_sr(q32, max(a - 7, 0)) == lo_code
            assert oracle.e2m1_sr(q32, min(b + 7, 65535)) == hi_code
        mean = (counts * vals).sum() / 65536.0
        step = 2.0 if abs(q32) >= 4 else (1.0 if abs(q32) >= 2 else 0.5)
        assert abs(mean - q32) <= step / 65536.0
        assert set(np.nonzero(counts)[0]) <= {lo_code, hi_code}
    # never clips below 6, saturates above
    assert oracle.e2m1_decode(oracle.e2m1_sr(6.0, 0)) == 6.0
    assert oracle.e2m1_decode(oracle.e2m1_sr(6.0001, 65535)) == 6.0
    # representable values are fixed points for every draw
    for code in range(16):
        for r in (0, 1, 40000, 65535):
            assert oracle.e2m1_sr(oracle.e2m1_decode(code), r) == code


def test_e4m3_sr_expectation_by_enumeration(oracle):
    # SR_FP8 of Algorithm 1 represents its argument exactly in expectation
    rng = np.random.default_rng(3)
    ts = np.concatenate([np.exp(rng.uniform(np.log(2.0 ** -9), np.log(440.0), 40)),
                         [2.0 ** -10, 0.001, 2.0 ** -6 * 0.99, 1.0, 1.03, 255.9, 447.9]]
                        ).astype(np.float32)
    for t in ts:
        t = float(t)
        lo_b = oracle.e4m3_sr(t, 0)
        hi_b = oracle.e4m3_sr(t, 2 ** 20 - 1)
        assert hi_b - lo_b in (0, 1)
        lo_v, hi_v = oracle.e4m3_decode(lo_b), oracle.e4m3_decode(hi_b)
        assert lo_v <= t <= max(hi_v, lo_v)
        if lo_b == hi_b:
            assert lo_v == t
            continue
        a, b = 0, 2 ** 20 - 1
        while b - a > 1:
            mid = (a + b) // 2
            if oracle.e4m3_sr(t, mid) == lo_b:
                a = mid
            else:
                b = mid
        p_up = (2 ** 20 - b) / 2.0 ** 20
        mean = lo_v + p_up * (hi_v - lo_v)
        assert abs(mean - t) <= (hi_v - lo_v) / 2.0 ** 20
    assert oracle.e4m3_sr(448.0, 0) == 0x7E and oracle.e4m3_sr(500.0, 2 ** 20 - 1) == 0x7E
    assert oracle.e4m3_sr(0.0, 123) == 0
    for b in range(127):
        for r in (0, 2 ** 20 - 1):
            assert oracle.e4m3_sr(oracle.e4m3_decode(b), r) == b
