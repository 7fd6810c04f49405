"""The exploratory NON-EXACT GEMM variants (qii_gemm_nvfp4_inexact).  They are measurement aids
outside the parity path, so they are not held to the exact GEMM's tolerance.  Checked here: each
variant computes what its description says (an emulation of the documented re-encoding of the
operands, written out below in numpy, followed by an exact product), and its distance from the
exact definition (the oracle's GEMM) has the size that re-encoding implies."""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii

from gpu_util import nv_to_dev

pytestmark = pytest.mark.gpu

E2M1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.0, -0.5, -1, -1.5, -2, -3, -4, -6], np.float64)


def e4m3_value(b):
    b = b.astype(np.int64)
    e, m = (b >> 3) & 15, b & 7
    return np.where(e == 0, m / 8.0 * 2.0 ** -6, (1 + m / 8.0) * 2.0 ** (e - 7.0))


def codes_of(q):
    c = q.codes
    return E2M1[np.stack([c & 15, c >> 4], -1).reshape(c.shape[0], -1)]


def reencode_fp8(q):
    """elements e2m1 * e4m3, per 32 of K: power-of-two scale putting the largest magnitude into
    [128, 256), elements rounded to E4M3 (nearest even) relative to it"""
    v = codes_of(q) * np.repeat(e4m3_value(q.scales), 16, axis=1)
    rows, K = v.shape
    blk = v.reshape(rows, K // 32, 32)
    mx = np.abs(blk).max(axis=2, keepdims=True)
    ex = np.where(mx > 0, np.floor(np.log2(np.where(mx > 0, mx, 1.0))) - 7, 0.0)
    r = torch.from_numpy((blk * 2.0 ** -ex).astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    return (r * 2.0 ** ex).reshape(rows, K)


def reencode_fp4_pow2(q):
    """codes as they are, each group's E4M3 scale replaced by the nearest power of two (1.5 and above
    round up; subnormals m * 2^-9: 1 -> 2^-9, 2 -> 2^-8, 3..5 -> 2^-7, 6..7 -> 2^-6; 0 stays 0)"""
    b = q.scales.astype(np.int64)
    e, m = (b >> 3) & 15, b & 7
    sub = np.select([m == 0, m == 1, m == 2, m <= 5], [-np.inf, -9.0, -8.0, -7.0], -6.0)
    p = np.where(e == 0, sub, e - 7.0 + (m >= 4))
    return codes_of(q) * np.repeat(np.where(np.isinf(p), 0.0, 2.0 ** np.where(np.isinf(p), 0.0, p)), 16, axis=1)


def run(qa, qb, variant, dtype=torch.float32, ldc=None):
    A, B = nv_to_dev(qa), nv_to_dev(qb)
    M, N, K = qa.rows, qb.rows, qa.cols
    ldc = ldc or N
    C = torch.full((M, ldc), 7.0, dtype=dtype, device="cuda")
    ws = torch.empty(max(256, qii.qii_gemm_inexact_workspace_bytes(M, N, K, variant)), dtype=torch.uint8, device="cuda")
    qii.qii_gemm_nvfp4_inexact(A, B, C[:, :N] if ldc != N else C, variant, ws)
    torch.cuda.synchronize()
    if ldc != N:
        assert bool((C[:, N:] == 7.0).all())
    return C[:, :N].float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (300, 200, 256), (513, 257, 384), (64, 700, 1024), (1024, 768, 2048)])
def test_inexact_variants_compute_what_they_say(oracle, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = (rng.standard_t(3, size=(M, K)) * 0.1).astype(np.float32)
    b = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    qa = oracle.quantize(a, oracle.RTN, rht_group=0)
    qb = oracle.quantize(b, oracle.MS_EDEN, rht_group=128, seed_sr=4)
    ts = float(qa.tensor_scale[0]) * float(qb.tensor_scale[0])
    exact, absum = oracle.gemm(qa, qb, with_abs=True)
    print(f"inexact gemm {M}x{N}x{K}", flush=True)
    for variant, reenc, tol, name in ((qii.INEXACT_FP8, reencode_fp8, 2e-3, "fp8"), (qii.INEXACT_FP4_POW2, reencode_fp4_pow2, 1e-5, "fp4_pow2")):
        if K % 64:
            continue
        ra, rb = reenc(qa), reenc(qb)
        ref = (ra @ rb.T) * ts
        ref_abs = (np.abs(ra) @ np.abs(rb).T) * abs(ts)
        got = run(qa, qb, variant, ldc=N + 8)
        # (the FP8 matrix instruction's own accumulation is not exact: a few 1e-4 of the sum of magnitudes)
        assert np.all(np.abs(got - ref) <= tol * ref_abs + 1e-30), (name, float(np.max(np.abs(got - ref) / (ref_abs + 1e-30))))
        rel = np.abs(got - exact) / (absum + 1e-30)
        print(f"  {name}: max |C - exact| / sum|a b| = {rel.max():.3g}, mean {rel.mean():.3g}", flush=True)
        # distance from the exact definition: FP8 rounds 6 significant bits to 4 (relative 2^-5 per
        # element at most, both operands); power-of-two scales are off by up to a factor 1.41
        assert rel.max() <= (0.07 if variant == qii.INEXACT_FP8 else 0.5)
        got16 = run(qa, qb, variant, dtype=torch.bfloat16)
        assert np.all(np.abs(got16 - ref) <= tol * ref_abs + 2.0 ** -8 * np.abs(ref) + 1e-30)


def test_inexact_gemm_rejects_bad_arguments():
    L = qii.lib()
    import ctypes
    from paper_2601_22813_amd.binding import _NVFP4
    a = _NVFP4(0x1000, 0x1000, 0x1000, 8, 96)
    b = _NVFP4(0x1000, 0x1000, 0x1000, 8, 96)
    assert L.qii_gemm_nvfp4_inexact(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 8, 1, 0x4000, 1 << 30, None) == 2   # K % 64
    a = _NVFP4(0x1000, 0x1000, 0x1000, 8, 64)
    b = _NVFP4(0x1000, 0x1000, 0x1000, 8, 64)
    assert L.qii_gemm_nvfp4_inexact(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 8, 5, 0x4000, 1 << 30, None) == 1   # variant
    assert L.qii_gemm_nvfp4_inexact(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 8, 0, None, 0, None) == 4           # workspace
    assert qii.qii_gemm_inexact_workspace_bytes(300, 200, 256, 0) == (2 + 1) * 4 * 18432
    assert qii.qii_gemm_inexact_workspace_bytes(300, 200, 256, 1) == (2 + 1) * 4 * 18432
