"""GPU parity of the quantizers on inputs built to reach the rarely taken branches of the tuned
kernels, byte for byte against the CPU oracle (through the C ABI):

  * tensors scaled by 2^-30, 2^30 and 2^-120: the abs-max leaves (2^-20, 2^20), so every division
    takes the full IEEE form instead of the short Newton sequences (and, at 2^-120, the tensor
    scale and many intermediates are binary32 denormals);
  * MS-EDEN tensors with one huge element: corrected group scales fall below 2^-6 (the E4M3
    subnormals, rounded stochastically on a uniform grid) and under-flow to byte 0;
  * exact ties of the element rounding: with a tensor scale of exactly 1 and a group scale of
    exactly 1 the rotated value itself is rounded, and the groups hold every binary32 within
    1024 ulps of the seven E2M1 midpoints, of the grid points, of 0 and the denormals;
  * exact ties of the scale rounding: group maxima placed on and next to all 126 E4M3 midpoints
    (subnormal ones included) and beyond the cap of 448;
  * the device self-test of the hardware conversions against their value-space rules.

Each case runs in the three kernel families: dense rows (contiguous source), columns (transposed
source whose quantized dimension is a multiple of 128) and the generic fallback.
"""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii
from paper_2601_22813_amd import synth

from gpu_util import assert_nv_equal, nv_to_dev, to_dev, ws

pytestmark = pytest.mark.gpu

MODES = [qii.RTN, qii.SR, qii.MS_EDEN, qii.RTN_46, qii.MS_EDEN_PH]
FAMILIES = ["rows", "cols", "generic"]


def quantize_logical(oracle, L, family, mode, rht_group, seed_rht, seed_sr, amax=None):
    """Quantize the logical R x C matrix L (groups along its rows) on the GPU in the given kernel
    family and on the oracle; returns (gpu NVFP4Tensor, oracle NVFP4).
    rows: L itself, contiguous.  cols / generic: the source is L^T and the call transposes it; the
    columns kernels take it when C is a multiple of 128 and R is even, otherwise the generic
    kernels do (callers pick shapes accordingly)."""
    R, C = L.shape
    if family == "rows":
        src, transpose = np.ascontiguousarray(L), False
    else:
        src, transpose = np.ascontiguousarray(L.T), True
        tuned = (C % 128 == 0) and (R % 2 == 0)
        assert tuned == (family == "cols"), f"shape {L.shape} does not select the {family} kernels"
    x = to_dev(src)
    out = qii.NVFP4Tensor.empty(R, C)
    out.codes.fill_(0xAB); out.scales.fill_(0xCD)
    am = None if amax is None else torch.tensor([amax], dtype=torch.float32, device="cuda")
    if mode == qii.MS_EDEN_PH:
        w = ws(qii.qii_quantize_posthoc_workspace_bytes(R, C))
    else:
        w = None if amax is not None else ws(256)
    qii.qii_quantize_nvfp4(x, transpose, mode, rht_group, seed_rht, seed_sr, am, out, w)
    ref = oracle.quantize(src, mode, transpose=transpose, rht_group=rht_group, seed_rht=seed_rht,
                          seed_sr=seed_sr, amax=amax)
    return out, ref


def family_shape(family, rht):
    """A logical shape (R, C) that selects the family; several chunks and a ragged tail."""
    if family == "rows":
        return (37, 384)
    if family == "cols":
        return (50, 256)
    return (51, 256) if rht else (18, 80)     # odd R (with rotation) / C not a multiple of 128


# ---------------------------------------------------------------- extreme magnitudes
@pytest.mark.parametrize("family", FAMILIES)
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("log2_scale", [-30, 30, -120])
def test_magnitudes_outside_the_short_division_range(oracle, log2_scale, mode, family):
    for rht in (128, 0):
        R, C = family_shape(family, rht)
        t = synth.bf16_bits_to_f32(synth.student_t_bf16((R, C), 3, 0.1, seed=31 + R))
        L = (t * np.float32(2.0 ** log2_scale)).astype(np.float32)
        assert np.all(np.isfinite(L)) and np.abs(L).max() > 0
        print(f"magnitude 2^{log2_scale} mode={mode} {family} rht={rht}", flush=True)
        out, ref = quantize_logical(oracle, L, family, mode, rht, 71, 72)
        assert_nv_equal(out, ref, f"2^{log2_scale} mode {mode} {family} rht {rht}")


@pytest.mark.parametrize("mode", MODES)
def test_magnitudes_bf16_rows_and_columns(oracle, mode):
    """The same with bf16 sources (the benchmark's dtype), whose exponent range is binary32's."""
    base = synth.bf16_bits_to_f32(synth.student_t_bf16((128, 256), 3, 0.1, seed=5))
    for log2_scale in (-30, 30, -120):
        xb = synth.f32_to_bf16_bits((base * np.float32(2.0 ** log2_scale)).astype(np.float32))
        for transpose in (False, True):
            R, C = (256, 128) if transpose else (128, 256)
            out = qii.NVFP4Tensor.empty(R, C)
            qii.qii_quantize_nvfp4(to_dev(xb), transpose, mode, 128, 5, 6, None, out,
                                   ws(qii.qii_quantize_posthoc_workspace_bytes(R, C)))
            ref = oracle.quantize(xb, mode, transpose=transpose, rht_group=128, seed_rht=5, seed_sr=6)
            assert_nv_equal(out, ref, f"bf16 2^{log2_scale} mode {mode} transpose {transpose}")


@pytest.mark.parametrize("family", FAMILIES)
def test_supplied_amax_on_both_sides_of_the_range_boundaries(oracle, family):
    """The short sequences are used for abs-max strictly inside (2^-20, 2^20): supply maxima on
    the boundaries and next to them."""
    R, C = family_shape(family, 128)
    L = synth.normal_f32((R, C), 1.0, 3)
    for amax in (2.0 ** 20, np.nextafter(np.float32(2.0 ** 20), np.float32(0)), 2.0 ** -20,
                 np.nextafter(np.float32(2.0 ** -20), np.float32(1))):
        scale = np.float32(amax) / np.abs(L).max() * np.float32(4.0)   # true maximum of the rotated tensor stays below
        for mode in (qii.RTN, qii.MS_EDEN, qii.RTN_46):
            out, ref = quantize_logical(oracle, (L * scale * np.float32(0.1)).astype(np.float32), family, mode, 128, 9, 10,
                                        amax=float(amax))
            assert_nv_equal(out, ref, f"amax {amax} mode {mode} {family}")


# ---------------------------------------------------------------- subnormal and vanishing scales
@pytest.mark.parametrize("family", FAMILIES)
@pytest.mark.parametrize("mode", [qii.MS_EDEN, qii.MS_EDEN_PH, qii.RTN, qii.SR])
def test_scales_below_the_normal_e4m3_range(oracle, mode, family):
    for rht in (0, 128):
        R, C = family_shape(family, rht)
        L = synth.normal_f32((R, C), 1.0, 77 + R)
        # group magnitudes fall by 2^-1/4 from one group of 16 to the next along every row, cycling
        # over 20 octaves, with a different phase per row; one element dominates the tensor
        g = (np.arange(C) // 16)[None, :] + 5 * np.arange(R)[:, None]
        L = (L * np.exp2(-0.25 * (g % 80)).astype(np.float32)).astype(np.float32)
        L[0, 0] = np.float32(3.0e3)
        out, ref = quantize_logical(oracle, L, family, mode, rht, 81, 82)
        sub = np.count_nonzero((ref.scales > 0) & (ref.scales < 8))
        zero = np.count_nonzero(ref.scales == 0)
        print(f"subnormal scales mode={mode} {family} rht={rht}: {sub} subnormal bytes, {zero} zero bytes "
              f"of {ref.scales.size}", flush=True)
        assert sub >= 4 and zero >= 4, "the input does not reach the branch under test"
        assert_nv_equal(out, ref, f"subnormal scales mode {mode} {family} rht {rht}")


# ---------------------------------------------------------------- exact ties of the element rounding
def tie_values():
    """Every binary32 within 1024 ulps of the E2M1 midpoints and grid points, of 6.0, of zero, the
    smallest denormals and a few tiny normals, both signs."""
    centres = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float32)
    offs = np.arange(-1024, 1025, dtype=np.int64)
    bits = (centres.view(np.uint32).astype(np.int64)[:, None] + offs[None, :]).reshape(-1)
    near = bits.astype(np.uint32).view(np.float32)
    small = np.arange(0, 1025, dtype=np.uint32).view(np.float32)                    # 0 and the first denormals
    tiny = (np.uint32(0x00800000) + np.arange(-512, 513)).astype(np.uint32).view(np.float32)   # around the smallest normal
    quarter = np.array([1e-30, 1e-20, 1e-10, 0.1, 0.2499, 0.2501, 5.9999, 6.0001], np.float32)
    v = np.concatenate([near, small, tiny, quarter])
    return np.concatenate([v, -v])


def tie_matrix(gmax, C, pad_to_even_rows=True):
    """Rows of C elements; every group of 16 holds 15 probe values and `gmax` (so that the group
    maximum, hence the group scale, is fixed), at a position that changes from group to group."""
    v = tie_values()
    v = v[np.abs(v) <= gmax]
    n_groups = -(-len(v) // 15)
    gpr = C // 16
    n_groups = -(-n_groups // gpr) * gpr
    R = n_groups // gpr
    if pad_to_even_rows and R % 2:
        R += 1
        n_groups += gpr
    vals = np.zeros(n_groups * 15, np.float32)
    vals[:len(v)] = v
    vals = vals.reshape(n_groups, 15)
    out = np.empty((n_groups, 16), np.float32)
    for gi in range(n_groups):
        pos = gi % 16
        out[gi] = np.insert(vals[gi], pos, np.float32(gmax))
    return out.reshape(R, C)


@pytest.mark.parametrize("family", FAMILIES)
def test_element_rounding_ties(oracle, family):
    """With tensor scale 1 and group scale 1 the rounded quantity is the stored value itself."""
    C = {"rows": 240, "cols": 128, "generic": 48}[family]
    s_eden = np.float32(96.0 / 17.0 / 0.93)
    s_sr = np.float32(96.0 / 17.0)
    cases = [
        (qii.RTN, np.float32(6.0), float(np.float32(6.0) * np.float32(448.0))),          # x32 = 2688 / (6 * 448) = 1
        (qii.RTN_46, np.float32(6.0), float(np.float32(6.0) * np.float32(256.0))),
        (qii.MS_EDEN, s_eden, float(s_eden * np.float32(256.0))),
        (qii.MS_EDEN_PH, s_eden, float(s_eden * np.float32(256.0))),
        (qii.SR, s_sr, float(s_sr * np.float32(448.0))),
    ]
    for mode, gmax, amax in cases:
        L = tie_matrix(gmax, C, pad_to_even_rows=(family == "cols"))
        if family == "generic" and L.shape[0] % 2 == 0 and C % 128 == 0:
            pytest.skip("shape would select the columns kernels")
        print(f"ties mode={mode} {family} shape={L.shape}", flush=True)
        out, ref = quantize_logical(oracle, L, family, mode, 0, 0, 91, amax=amax)
        if mode in (qii.RTN, qii.MS_EDEN, qii.MS_EDEN_PH, qii.SR):
            assert ref.tensor_scale[0] == 1.0
        if mode in (qii.RTN, qii.SR):
            assert np.all(ref.scales == 0x38), "group scales are meant to be exactly 1"
        assert_nv_equal(out, ref, f"element ties mode {mode} {family}")


# ---------------------------------------------------------------- exact ties of the scale rounding
def e4m3_values():
    b = np.arange(127)
    e, m = b >> 3, b & 7
    return np.where(e == 0, m / 8.0 * 2.0 ** -6, (1 + m / 8.0) * np.exp2(e - 7.0)).astype(np.float64)


@pytest.mark.parametrize("family", FAMILIES)
def test_scale_rounding_ties_and_saturation(oracle, family):
    """RTN with amax = 2688 gives x32 = 1 and a scale quotient of gmax / 6: group maxima are placed
    so that the quotient lands on every E4M3 midpoint and 1..2 ulps beside it, and beyond 448."""
    C = {"rows": 208, "cols": 128, "generic": 48}[family]
    grid = e4m3_values()
    mids = ((grid[:-1] + grid[1:]) / 2).astype(np.float32)             # exact in binary32
    rng = np.random.default_rng(4)
    for mode, level, cap in ((qii.RTN, 6.0, 448.0), (qii.RTN_46, 6.0, 256.0), (qii.RTN_46, 4.0, 256.0),
                             (qii.SR, float(np.float32(96.0 / 17.0)), 448.0),
                             (qii.MS_EDEN, float(np.float32(96.0 / 17.0 / 0.93)), 256.0)):
        lv = np.float32(level)
        targets = []
        for k in (-2, -1, 0, 1, 2):
            q = (mids.view(np.uint32).astype(np.int64) + k).astype(np.uint32).view(np.float32)
            targets.append(q * lv)                                       # gmax with gmax / level = q (up to one rounding)
        targets.append(np.array([448.0, 449.0, 460.0, 480.0, 1000.0, 1e6], np.float32) * lv)
        gm = np.concatenate(targets).astype(np.float32)
        gm = gm[gm > 0]
        gpr = C // 16
        n_groups = -(-len(gm) // gpr) * gpr
        if family == "cols" and (n_groups // gpr) % 2:
            n_groups += gpr
        g = np.zeros(n_groups, np.float32)
        g[:len(gm)] = gm
        body = rng.uniform(-1, 1, (n_groups, 16)).astype(np.float32) * (g[:, None] * np.float32(0.9))
        body[np.arange(n_groups), np.arange(n_groups) % 16] = g * np.where(np.arange(n_groups) % 2, -1, 1).astype(np.float32)
        L = body.reshape(n_groups // gpr, C)
        if family == "generic" and L.shape[0] % 2 == 0 and C % 128 == 0:
            pytest.skip("shape would select the columns kernels")
        amax = float(np.float32(6.0 if mode == qii.RTN_46 else level) * np.float32(cap))    # x32 = 1
        print(f"scale ties mode={mode} level={level} {family} shape={L.shape}", flush=True)
        out, ref = quantize_logical(oracle, L, family, mode, 0, 0, 93, amax=amax)
        assert ref.tensor_scale[0] == 1.0
        if mode == qii.RTN:
            assert np.count_nonzero(ref.scales == 0x7E) >= 6
        assert_nv_equal(out, ref, f"scale ties mode {mode} level {level} {family}")


# ---------------------------------------------------------------- hardware conversions
def test_hardware_conversions_match_their_value_space_rules():
    counts = torch.full((8,), -1, dtype=torch.int64, device="cuda")
    qii.qii_selftest_conversions(counts)
    torch.cuda.synchronize()
    got = counts.cpu().tolist()
    names = ["fp4 encode", "e4m3 encode", "fp4 decode", "fp4 x e4m3 -> f16", "division by constant",
             "short division", "e4m3 decode", "reciprocals"]
    print("self-test mismatch counts:", dict(zip(names, got)), flush=True)
    assert got == [0] * 8, dict(zip(names, got))


def test_requantize_with_extreme_tensor_scale(oracle):
    """The NVFP4-source loaders (dequantize on load) with a saved tensor whose tensor scale puts the
    dequantized values outside the short-division range."""
    rng = np.random.default_rng(12)
    rows, cols = 256, 128
    for ts in (2.0 ** -40, 2.0 ** 35):
        saved = oracle.NVFP4(rng.integers(0, 256, (rows, cols // 2)).astype(np.uint8),
                             rng.integers(0x20, 0x60, (rows, cols // 16)).astype(np.uint8),
                             np.array([ts], np.float32))
        dev_saved = nv_to_dev(saved)
        for transpose, shape in ((True, (cols, rows)), (False, (rows, cols))):
            for mode in (qii.MS_EDEN, qii.MS_EDEN_PH):
                out = qii.NVFP4Tensor.empty(*shape)
                qii.qii_requantize_nvfp4(dev_saved, transpose, mode, 128, 61, 62, None, out,
                                         ws(qii.qii_quantize_posthoc_workspace_bytes(*shape)))
                ref = oracle.requantize(saved, mode, transpose=transpose, seed_rht=61, seed_sr=62)
                assert_nv_equal(out, ref, f"requantize ts {ts} mode {mode} transpose {transpose}")
