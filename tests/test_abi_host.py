"""Host-only checks of the C ABI: the library loads, exports every symbol that
include/qii.h declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def libqii():
    from paper_2601_22813_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(force=True)
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qii.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qii_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(libqii):
    names = declared_symbols()
    assert len(names) >= 16
    L = libqii.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(libqii.EXPORTS) == names


def test_host_helpers(libqii, oracle):
    assert libqii.qii_version() >= 1
    for seed in (0, 7, 2 ** 63 + 5):
        for i in range(6):
            assert libqii.qii_derive_seed(seed, i) == oracle.derive_seed(seed, i)
    assert libqii.qii_quantize_workspace_bytes() == 256
    need = libqii.qii_linear_bwd_workspace_bytes(256, 128, 384)
    # four NVFP4 operands: codes, and scale bytes with room for the row count rounded up to 256
    up = lambda r: (r + 255) // 256 * 256
    payload = sum(r * c // 2 + up(r) * c // 16 for r, c in ((256, 384), (128, 384), (384, 256), (128, 256)))
    gemm_ws = max(libqii.qii_gemm_workspace_bytes(256, 128, 384), libqii.qii_gemm_workspace_bytes(384, 128, 256))
    assert payload + gemm_ws <= need <= payload + gemm_ws + 16 * 256
    # re-tiled scale bytes of both operands, rows padded to 256; nothing when K is not a multiple of 256
    assert libqii.qii_gemm_workspace_bytes(300, 200, 512) == (512 + 256) * 512 // 16
    assert libqii.qii_gemm_workspace_bytes(300, 200, 384) == 0
    # whole rounds of 256 tiles need the scale bytes only; an incomplete last round whose tiles are
    # shared between blocks adds one 256 KiB partial tile per sharing block and shared tile
    scales = lambda M, N, K: (up(M) + up(N)) * K // 16
    assert libqii.qii_gemm_workspace_bytes(16384, 8192, 2048) == scales(16384, 8192, 2048)       # 2048 tiles
    assert libqii.qii_gemm_workspace_bytes(4096, 4096, 32768) == scales(4096, 4096, 32768)       # 256 tiles
    extra = libqii.qii_gemm_workspace_bytes(2048, 2048, 32768) - scales(2048, 2048, 32768)       # 64 tiles, long K
    assert extra == (256 + 64) * 256 * 256 * 4
    extra = libqii.qii_gemm_workspace_bytes(11264, 2048, 16384) - scales(11264, 2048, 16384)     # 352 tiles: 96 shared
    assert extra == (256 + 96) * 256 * 256 * 4
    assert libqii.qii_gemm_workspace_bytes(2048, 5632, 16384) == scales(2048, 5632, 16384)       # 176 tiles: stays plain
    assert libqii.qii_gemm_workspace_bytes(512, 512, 1024) == scales(512, 512, 1024)             # short K: stays plain
    L = libqii.lib()
    assert L.qii_status_string(0) == b"QII_OK" and L.qii_status_string(2) == b"QII_BAD_SHAPE"


def test_bad_arguments_are_rejected_without_a_device(libqii):
    L = libqii.lib()
    out = libqii.binding._NVFP4(8, 8, 8, 4, 120) if hasattr(libqii, "binding") else None
    from paper_2601_22813_amd.binding import _NVFP4
    out = _NVFP4(0x1000, 0x1000, 0x1000, 4, 120)
    # quantized dimension not a multiple of 16
    st = L.qii_quantize_nvfp4(0x1000, 1, 4, 120, 120, 0, 0, 0, 0, 0, None, ctypes.byref(out), None, 0, None)
    assert st == 2 and b"multiple" in L.qii_last_error()
    # rotation needs multiples of 128
    out = _NVFP4(0x1000, 0x1000, 0x1000, 4, 64)
    st = L.qii_quantize_nvfp4(0x1000, 1, 4, 64, 64, 0, 2, 128, 0, 0, None, ctypes.byref(out), None, 0, None)
    assert st == 2
    # bad mode, bad dtype, null input, misaligned input
    out = _NVFP4(0x1000, 0x1000, 0x1000, 4, 128)
    assert L.qii_quantize_nvfp4(0x1000, 1, 4, 128, 128, 0, 9, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 1
    assert L.qii_quantize_nvfp4(0x1000, 5, 4, 128, 128, 0, 2, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 1
    assert L.qii_quantize_nvfp4(None, 1, 4, 128, 128, 0, 2, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 1
    assert L.qii_quantize_nvfp4(0x1002, 1, 4, 128, 128, 0, 2, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 1
    assert L.qii_quantize_nvfp4(0x1001, 1, 128, 4, 4, 1, 2, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 1
    # output shape mismatch (transpose swaps it)
    assert L.qii_quantize_nvfp4(0x1000, 1, 4, 128, 128, 1, 0, 0, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 2
    # no amax and no workspace
    assert L.qii_quantize_nvfp4(0x1000, 1, 4, 128, 128, 0, 2, 128, 0, 0, None, ctypes.byref(out), None, 0, None) == 4
    # GEMM: inner dimensions differ / K not a multiple of 16 / ldc < N / bad dtype / null or misaligned C
    a = _NVFP4(0x1000, 0x1000, 0x1000, 8, 64)
    b = _NVFP4(0x1000, 0x1000, 0x1000, 8, 128)
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 8, None, 0, None) == 2
    a = _NVFP4(0x1000, 0x1000, 0x1000, 8, 40)
    b = _NVFP4(0x1000, 0x1000, 0x1000, 8, 40)
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 8, None, 0, None) == 2
    a = _NVFP4(0x1000, 0x1000, 0x1000, 8, 48)
    b = _NVFP4(0x1000, 0x1000, 0x1000, 8, 48)
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), 0x3000, 0, 7, None, 0, None) == 2
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), 0x3000, 7, 8, None, 0, None) == 1
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), None, 0, 8, None, 0, None) == 1
    assert L.qii_gemm_nvfp4(ctypes.byref(a), ctypes.byref(b), 0x3002, 0, 8, None, 0, None) == 1
    # linear_bwd: workspace too small
    xq = _NVFP4(0x1000, 0x1000, 0x1000, 256, 128)
    wq = _NVFP4(0x1000, 0x1000, 0x1000, 384, 128)
    assert L.qii_linear_bwd(0x1000, 1, ctypes.byref(xq), ctypes.byref(wq), 0, 0x1000, 0x1000, 1, 0x1000, 16, None) == 4
    # empty tensors are accepted and do nothing
    out = _NVFP4(None, None, None, 0, 128)
    assert L.qii_quantize_nvfp4(None, 1, 0, 128, 128, 0, 2, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 0


def test_new_modes_and_layer_variants_reject_bad_arguments(libqii):
    L = libqii.lib()
    from paper_2601_22813_amd.binding import _NVFP4
    out = _NVFP4(0x1000, 0x1000, 0x1000, 4, 128)
    # post hoc scheme: needs its per-group buffer even when the abs-max is supplied
    assert L.qii_quantize_nvfp4(0x1000, 1, 4, 128, 128, 0, 4, 128, 0, 0, 0x2000, ctypes.byref(out), None, 0, None) == 4
    assert L.qii_quantize_nvfp4(0x1000, 1, 4, 128, 128, 0, 4, 128, 0, 0, 0x2000, ctypes.byref(out), 0x4000, 256, None) == 4
    assert libqii.qii_quantize_posthoc_workspace_bytes(4, 128) == 16384 + 256    # running-maximum region + 32 floats, padded
    assert libqii.qii_quantize_posthoc_workspace_bytes(8192, 8192) == 16384 + 8192 * 512 * 4
    # the layer variants only take the modes that make sense for their pass
    xq = _NVFP4(0x1000, 0x1000, 0x1000, 256, 128)
    wq = _NVFP4(0x1000, 0x1000, 0x1000, 384, 128)
    big = 1 << 30
    assert L.qii_linear_fwd_mode(0x1000, 0x1000, 1, 256, 128, 384, 2, None, None, 0x1000, 1, ctypes.byref(xq), ctypes.byref(wq), 0x1000, big, None) == 1
    assert L.qii_linear_bwd_mode(0x1000, 1, ctypes.byref(xq), ctypes.byref(wq), 0, 1, 0x1000, 0x1000, 1, 0x1000, big, None) == 1
    assert L.qii_linear_bwd_mode(0x1000, 1, ctypes.byref(xq), ctypes.byref(wq), 0, 4, 0x1000, 0x1000, 1, 0x1000, 16, None) == 4
    plain = libqii.qii_linear_bwd_mode_workspace_bytes(256, 128, 384, 2)
    assert plain == libqii.qii_linear_bwd_workspace_bytes(256, 128, 384)
    # four 16 KiB running-maximum regions instead of four slots, and one per-group f32 buffer for each of Q(E), Q(E^T)
    assert libqii.qii_linear_bwd_mode_workspace_bytes(256, 128, 384, 4) == plain + 4 * (16384 - 256) + 2 * 256 * 384 // 16 * 4
    assert libqii.qii_quantize_pair_workspace_bytes(256, 384, 2) == 512
    assert libqii.qii_quantize_pair_workspace_bytes(256, 384, 4) == 2 * 16384 + 2 * 256 * 384 // 16 * 4


def test_layer_passes_validate_everything_before_the_first_launch(libqii):
    """No device is present here, so any launch would come back as QII_HIP_ERROR (5): getting the
    argument status instead shows that the whole pass is checked before anything is enqueued."""
    L = libqii.lib()
    from paper_2601_22813_amd.binding import _NVFP4
    T, d_in, d_out = 256, 128, 384
    xq = _NVFP4(0x10000, 0x20000, 0x30000, T, d_in)
    wq = _NVFP4(0x40000, 0x50000, 0x60000, d_out, d_in)
    big = 1 << 30
    fwd = lambda X=0x1000, W=0x2000, dt=1, Y=0x3000, ydt=1, xq_=xq, wq_=wq, ws=0x100000, wsb=big: L.qii_linear_fwd_mode(
        X, W, dt, T, d_in, d_out, 0, None, None, Y, ydt, ctypes.byref(xq_), ctypes.byref(wq_), ws, wsb, None)
    assert fwd(Y=None) == 1 and b"null C" in L.qii_last_error()
    assert fwd(ydt=9) == 1
    assert fwd(X=None) == 1
    assert fwd(W=None) == 1
    assert fwd(dt=9) == 1
    assert fwd(xq_=_NVFP4(0x10000, 0x20000, 0x30000, T, d_in + 16)) == 2
    assert fwd(wq_=_NVFP4(0x40000, 0x50000, None, d_out, d_in)) == 1
    assert fwd(wsb=16) == 4
    assert fwd(ws=0x100010) == 4
    bwd = lambda dY=0x1000, dt=1, dX=0x3000, dW=0x5000, gdt=1, xq_=xq, wq_=wq, ws=0x100000, wsb=big, mode=2: L.qii_linear_bwd_mode(
        dY, dt, ctypes.byref(xq_), ctypes.byref(wq_), 0, mode, dX, dW, gdt, ws, wsb, None)
    assert bwd(dY=None) == 1
    assert bwd(dt=3) == 1
    assert bwd(dX=None) == 1
    assert bwd(dW=None) == 1 and b"dW" in L.qii_last_error()
    assert bwd(gdt=5) == 1
    assert bwd(dX=0x3001) == 1
    assert bwd(wq_=_NVFP4(0x40000, 0x50000, 0x60000, d_out, d_in + 16)) == 2
    assert bwd(xq_=_NVFP4(0x10000, 0x20000, 0x30000, T + 64, d_in)) == 2      # T not a multiple of 128
    assert bwd(wsb=16) == 4
    assert bwd(mode=4, wsb=libqii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, 4) - 1) == 4


def test_binding_refuses_strided_layer_tensors(libqii):
    import torch
    X = torch.zeros((8, 64), dtype=torch.bfloat16)[:, :32]      # row stride 64, 32 columns used
    W = torch.zeros((16, 32), dtype=torch.bfloat16)
    Y = torch.zeros((8, 16), dtype=torch.bfloat16)
    xq, wq = libqii.NVFP4Tensor.empty(8, 32, device="cpu"), libqii.NVFP4Tensor.empty(16, 32, device="cpu")
    with pytest.raises(libqii.QiiError, match="contiguous"):
        libqii.qii_linear_fwd(X, W, Y, xq, wq, torch.zeros(4096, dtype=torch.uint8))
    dX, dW = torch.zeros((8, 32), dtype=torch.bfloat16), torch.zeros((16, 32), dtype=torch.float32)
    with pytest.raises(libqii.QiiError, match="same dtype"):
        libqii.qii_linear_bwd(Y, xq, wq, 0, dX, dW, torch.zeros(4096, dtype=torch.uint8))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
