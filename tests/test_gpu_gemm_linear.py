"""GPU parity of the block-scaled GEMM and of the layer passes against the CPU oracle.

Tolerance (GEMM): the kernel forms every product e2m1*e4m3 x e2m1*e4m3 exactly and
accumulates in f32, so |C_gpu - C_ref| <= 1e-5 * sum_k |A_hat B_hat| covers the f32
accumulation (K <= 16384 terms added in blocks of 16 by the matrix unit, relative error per
addition 2^-24) plus the one rounding of the epilogue scaling; bf16 outputs add one bf16
rounding, 2^-8 |C_ref|."""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii
from paper_2601_22813_amd import synth

from gpu_util import assert_nv_equal, bf16_to_f64, nv_to_dev, to_dev, ws

pytestmark = pytest.mark.gpu

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, -0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0])


def gemm_gpu(qa, qb, dtype, ldc=None, use_ws=True):
    """With a workspace the fast kernel runs (when K is a multiple of 256); without, the fallbacks."""
    M, N = qa.rows, qb.rows
    ldc = ldc or N
    C = torch.full((M, ldc), float("nan"), dtype=dtype, device="cuda")
    w = ws(qii.qii_gemm_workspace_bytes(M, N, qa.cols)) if use_ws else None
    if w is not None:
        w.fill_(0x7F)   # a scale byte the library never writes: stale workspace must not leak in
    qii.qii_gemm_nvfp4(nv_to_dev(qa), nv_to_dev(qb), C, w)
    torch.cuda.synchronize()
    return C[:, :N].float().cpu().numpy().astype(np.float64)


def check(C, ref, absum, bf16):
    tol = 1e-5 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-30
    err = np.abs(C - ref)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), f"worst at {worst}: gpu {C[worst]} ref {ref[worst]} tol {tol[worst] if np.ndim(tol) else tol}"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gemm_256_cubed_config(oracle, dtype):
    X = synth.normal_f32((256, 256), 1.0, 0)
    W = synth.normal_f32((256, 256), 0.02, 1)
    for mode in (oracle.RTN, oracle.SR, oracle.MS_EDEN):
        qa = oracle.quantize(X, mode, seed_rht=0, seed_sr=0)
        qb = oracle.quantize(W, mode, seed_rht=0, seed_sr=1)
        ref, absum = oracle.gemm(qa, qb, with_abs=True)
        check(gemm_gpu(qa, qb, dtype), ref, absum, dtype == torch.bfloat16)
        check(gemm_gpu(qa, qb, dtype, use_ws=False), ref, absum, dtype == torch.bfloat16)


@pytest.mark.parametrize("M,N,K", [(300, 200, 160), (1, 1, 32), (513, 257, 384), (64, 700, 1024),
                                   (256, 256, 96), (300, 520, 512), (1024, 768, 2048)])
def test_gemm_ragged_shapes(oracle, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = (rng.standard_t(3, size=(M, K)) * 0.1).astype(np.float32)
    b = rng.standard_normal((N, K)).astype(np.float32)
    qa = oracle.quantize(a, oracle.RTN, rht_group=0)
    qb = oracle.quantize(b, oracle.SR, rht_group=0, seed_sr=4)
    ref, absum = oracle.gemm(qa, qb, with_abs=True)
    print(f"gemm {M}x{N}x{K}", flush=True)
    check(gemm_gpu(qa, qb, torch.float32, ldc=N + 8), ref, absum, False)
    check(gemm_gpu(qa, qb, torch.bfloat16), ref, absum, True)
    check(gemm_gpu(qa, qb, torch.bfloat16, ldc=N + 3, use_ws=False), ref, absum, True)


@pytest.mark.parametrize("M,N,K", [(512, 512, 8192), (300, 520, 4096), (1280, 256, 6144), (256, 256, 4096), (6100, 2800, 4096)])
def test_gemm_shares_the_tiles_of_an_incomplete_round(oracle, M, N, K):
    """Tiles beyond the last full round of 256 (all of them when there are fewer) are shared between
    blocks: contiguous ranges of K tiles, partial tiles in the workspace, added up in a fixed order.
    Same tolerance, same result on a repeated call, and the emitted max |C| is that of the stored
    values; without room for the partial tiles the plain path runs.  The shapes cover 4 / 6 / 5 / 1
    tiles (block counts 32, 24, 24, 4; an odd tile count with ranges that span two tiles; ragged
    edges) and 264 tiles (one full round, then 8 shared tiles)."""
    rng = np.random.default_rng(M + N + K)
    a = (rng.standard_t(3, size=(M, K)) * 0.1).astype(np.float32)
    b = rng.standard_normal((N, K)).astype(np.float32)
    qa = oracle.quantize(a, oracle.RTN, rht_group=0)
    qb = oracle.quantize(b, oracle.MS_EDEN, rht_group=128, seed_sr=4)
    ref, absum = oracle.gemm(qa, qb, with_abs=True)
    need = qii.qii_gemm_workspace_bytes(M, N, K)
    rem = (-(-M // 256) * -(-N // 256)) % 256
    assert need > (M + 255) // 256 * 256 * (K // 16) + (N + 255) // 256 * 256 * (K // 16) + 2 * rem * 65536 * 4 - 1   # room for >= 2 partial tiles per shared tile
    print(f"gemm {M}x{N}x{K}, workspace {need}", flush=True)
    c1 = gemm_gpu(qa, qb, torch.float32, ldc=N + 8)
    check(c1, ref, absum, False)
    assert np.array_equal(c1, gemm_gpu(qa, qb, torch.float32, ldc=N + 8))
    check(gemm_gpu(qa, qb, torch.bfloat16), ref, absum, True)
    A, B = nv_to_dev(qa), nv_to_dev(qb)
    for dtype in (torch.float32, torch.bfloat16):
        C = torch.empty((M, N), dtype=dtype, device="cuda")
        amax = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        qii.qii_gemm_nvfp4_amax(A, B, C, amax, ws(need))
        torch.cuda.synchronize()
        assert float(amax[0]) == float(C.float().abs().max())
    # a workspace that only holds the re-tiled scales: one block per tile
    small = ws((M + 255) // 256 * 256 * (K // 16) + (N + 255) // 256 * 256 * (K // 16))
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    qii.qii_gemm_nvfp4(A, B, C, small)
    torch.cuda.synchronize()
    check(C.cpu().numpy().astype(np.float64), ref, absum, False)


def test_gemm_unit_scales_is_exact(oracle):
    # every scale byte 1.0 and tensor scale 1: all partial sums are multiples of 1/4 below 2^24,
    # so the f32 result must equal the integer result exactly whatever the accumulation order
    rng = np.random.default_rng(8)
    M, N, K = 320, 288, 2048
    qa = oracle.NVFP4(rng.integers(0, 256, (M, K // 2)).astype(np.uint8), np.full((M, K // 16), 0x38, np.uint8), np.ones(1, np.float32))
    qb = oracle.NVFP4(rng.integers(0, 256, (N, K // 2)).astype(np.uint8), np.full((N, K // 16), 0x38, np.uint8), np.ones(1, np.float32))
    C = gemm_gpu(qa, qb, torch.float32)
    unpack = lambda c: np.stack([c & 15, c >> 4], -1).reshape(c.shape[0], -1)
    ia = np.rint(E2M1[unpack(qa.codes)] * 2).astype(np.int64)
    ib = np.rint(E2M1[unpack(qb.codes)] * 2).astype(np.int64)
    assert np.array_equal(C * 4, (ia @ ib.T).astype(np.float64))


def test_gemm_all_scale_bytes_and_codes(oracle):
    # every E4M3 byte (subnormals included) against every FP4 code: dequantization is exact
    K = 128
    scales = np.arange(0, 127, dtype=np.uint8)
    M = 127
    a_codes = np.tile(np.array([0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE], np.uint8), (M, K // 16))
    qa = oracle.NVFP4(a_codes, np.repeat(scales[:, None], K // 16, 1), np.array([1.0], np.float32))
    b_codes = np.zeros((16, K // 2), np.uint8)
    for n in range(16):      # B row n picks element n of every group with value 1.0 (code 2)
        for g in range(K // 16):
            b_codes[n, (g * 16 + n) // 2] = 2 << (4 * (n & 1))
    qb = oracle.NVFP4(b_codes, np.full((16, K // 16), 0x38, np.uint8), np.array([1.0], np.float32))
    C = gemm_gpu(qa, qb, torch.float32)
    ref = oracle.gemm(qa, qb)
    assert np.array_equal(C, ref)


def test_linear_forward_and_backward(oracle):
    T, d_in, d_out = 512, 256, 384
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=2)
    X, W, E = to_dev(Xb), to_dev(Wb), to_dev(Eb)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    qii.qii_linear_fwd(X, W, Y, Xq, Wq, ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out)))
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    assert_nv_equal(Xq, oXq, "saved X")
    assert_nv_equal(Wq, oWq, "saved W")
    ref, absum = oracle.gemm(oXq, oWq, with_abs=True)
    check(bf16_to_f64(Y), ref, absum, True)
    for seed in (0, 12345):
        dX = torch.empty((T, d_in), dtype=torch.float32, device="cuda")
        dW = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
        qii.qii_linear_bwd(E, Xq, Wq, seed, dX, dW, ws(qii.qii_linear_bwd_workspace_bytes(T, d_in, d_out)))
        Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, oXq, oWq, seed)
        ref, absum = oracle.gemm(Eq, WTq, with_abs=True)
        torch.cuda.synchronize()
        check(dX.cpu().numpy().astype(np.float64), ref, absum, False)
        ref, absum = oracle.gemm(ETq, XTq, with_abs=True)
        check(dW.cpu().numpy().astype(np.float64), ref, absum, False)


@pytest.mark.parametrize("T,d_in,d_out", [(256, 384, 512), (384, 208, 512), (512, 384, 640), (128, 64, 128)])
def test_linear_backward_with_post_hoc_range_alignment(oracle, T, d_in, d_out):
    """Backward pass of Sec. 5 with the four quantizers in the two-kernel form of Sec. 7.  (Where a
    GEMM's inner dimension, d_out or T, is a multiple of 256 the scales pass writes the scale bytes
    in the GEMM kernel's tiled layout; the shapes cover both, one and none of the two GEMMs.)"""
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=8)
    E = to_dev(Eb)
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    Xq, Wq = nv_to_dev(oXq), nv_to_dev(oWq)
    seed = 77
    dX = torch.empty((T, d_in), dtype=torch.float32, device="cuda")
    dW = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    w = ws(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH))
    qii.qii_linear_bwd_mode(E, Xq, Wq, seed, qii.MS_EDEN_PH, dX, dW, w)
    Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, oXq, oWq, seed, mode=oracle.MS_EDEN_PH)
    ref, absum = oracle.gemm(Eq, WTq, with_abs=True)
    torch.cuda.synchronize()
    check(dX.cpu().numpy().astype(np.float64), ref, absum, False)
    ref, absum = oracle.gemm(ETq, XTq, with_abs=True)
    check(dW.cpu().numpy().astype(np.float64), ref, absum, False)
    with pytest.raises(qii.QiiError):
        qii.qii_linear_bwd_mode(E, Xq, Wq, seed, qii.SR, dX, dW, w)


def test_linear_forward_with_four_over_six(oracle):
    """Forward pass of Sec. 5 with the 4/6 choice of Sec. 4.1 on X and W; other modes are refused."""
    T, d_in, d_out = 384, 512, 256
    Xb, Wb, _ = synth.linear_layer_bf16(T, d_in, d_out, seed=5)
    X, W = to_dev(Xb), to_dev(Wb)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.float32, device="cuda")
    w = ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out))
    qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y, Xq, Wq, w)
    oXq, oWq = oracle.linear_fwd(Xb, Wb, mode=oracle.RTN_46)
    assert_nv_equal(Xq, oXq, "saved X (4/6)")
    assert_nv_equal(Wq, oWq, "saved W (4/6)")
    ref, absum = oracle.gemm(oXq, oWq, with_abs=True)
    torch.cuda.synchronize()
    check(Y.cpu().numpy().astype(np.float64), ref, absum, False)
    with pytest.raises(qii.QiiError):
        qii.qii_linear_fwd_mode(X, W, qii.MS_EDEN, Y, Xq, Wq, w)
    # with the two maxima supplied by the caller the result is the same
    ax = torch.zeros(1, dtype=torch.float32, device="cuda"); aw = torch.zeros(1, dtype=torch.float32, device="cuda")
    qii.qii_absmax(X, False, 0, 0, ax); qii.qii_absmax(W, False, 0, 0, aw)
    Xq2, Wq2 = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y2 = torch.empty_like(Y)
    qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y2, Xq2, Wq2, w, amax_x=ax, amax_w=aw)
    assert_nv_equal(Xq2, oXq, "saved X (4/6, supplied maximum)")
    assert_nv_equal(Wq2, oWq, "saved W (4/6, supplied maximum)")
    assert torch.equal(Y2, Y)


@pytest.mark.parametrize("T,d_in,d_out,zero_x", [(320, 768, 272, False), (320, 384, 272, False), (320, 768, 272, True)])
def test_linear_forward_scale_layouts(oracle, T, d_in, d_out, zero_x):
    """With d_in a multiple of 256 the forward quantizers also write their scale bytes in the GEMM
    kernel's tiled layout (ragged row counts here: 320 and 272 rows in tiles of 256); otherwise the
    GEMM reads the row-major bytes.  Saved operands and Y must match either way, also for an all-zero
    X, whose quantizer takes a separate path."""
    Xb, Wb, _ = synth.linear_layer_bf16(T, d_in, d_out, seed=11)
    if zero_x:
        Xb = np.zeros_like(Xb)
    X, W = to_dev(Xb), to_dev(Wb)
    for mode, omode in ((qii.RTN, oracle.RTN), (qii.RTN_46, oracle.RTN_46)):
        Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
        Y = torch.full((T, d_out), 7.0, dtype=torch.float32, device="cuda")
        qii.qii_linear_fwd_mode(X, W, mode, Y, Xq, Wq, ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out)))
        oXq, oWq = oracle.linear_fwd(Xb, Wb, mode=omode)
        assert_nv_equal(Xq, oXq, "saved X")
        assert_nv_equal(Wq, oWq, "saved W")
        ref, absum = oracle.gemm(oXq, oWq, with_abs=True)
        torch.cuda.synchronize()
        check(Y.cpu().numpy().astype(np.float64), ref, absum, False)
        if zero_x:
            assert float(Y.abs().max()) == 0.0


def test_layer_passes_replay_from_a_hip_graph(oracle):
    """Nothing in the library allocates, synchronises or uses memset nodes, so a forward + backward
    pass can be captured once and replayed; every replay (with eager work and synchronisations in
    between) must reproduce the eager results bit for bit, on fresh inputs written into the same
    buffers."""
    T, d_in, d_out = 256, 256, 384
    X = torch.empty((T, d_in), dtype=torch.bfloat16, device="cuda")
    W = torch.empty((d_out, d_in), dtype=torch.bfloat16, device="cuda")
    E = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.float32, device="cuda")
    dX = torch.empty((T, d_in), dtype=torch.float32, device="cuda")
    dW = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    wf = ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out))
    wb = ws(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH))

    def run():
        qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y, Xq, Wq, wf)
        qii.qii_linear_bwd_mode(E, Xq, Wq, 5, qii.MS_EDEN_PH, dX, dW, wb)

    def fill(seed):
        Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=seed)
        X.copy_(to_dev(Xb)); W.copy_(to_dev(Wb)); E.copy_(to_dev(Eb))

    fill(100)
    run()                       # warm-up outside the capture (function attributes, module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.current_stream().wait_stream(side)
    for seed in (101, 102, 103):
        fill(seed)
        run()
        torch.cuda.synchronize()
        want = [t.clone() for t in (Y, dX, dW, Xq.codes, Xq.scales, Wq.codes, Wq.scales)]
        for t in (Y, dX, dW):
            t.zero_()
        Xq.codes.zero_(); Wq.scales.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (Y, dX, dW, Xq.codes, Xq.scales, Wq.codes, Wq.scales)
        for k, (g, w_) in enumerate(zip(got, want)):
            assert torch.equal(g, w_), f"replay with seed {seed}: tensor {k} differs from the eager run"


@pytest.mark.parametrize("M,N,K,use_ws", [(300, 200, 160, False), (513, 257, 384, False), (300, 520, 512, True),
                                          (1024, 768, 2048, True), (64, 70, 48, False), (256, 256, 256, True)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gemm_emits_the_abs_max_of_what_it_stores(oracle, M, N, K, use_ws, dtype):
    """max |C| out of the GEMM's epilogue (the abs-max the consumer's quantizer needs, App. D): it
    must equal the maximum over the stored matrix bit for bit, in all three kernels, and entries of
    the padded tile beyond M x N must not leak into it.  K = 48 also covers an inner dimension that
    is a multiple of 16 but not of 32."""
    rng = np.random.default_rng(M * 7 + N + K)
    a = (rng.standard_t(3, size=(M, K)) * 0.1).astype(np.float32)
    b = rng.standard_normal((N, K)).astype(np.float32)
    qa = oracle.quantize(a, oracle.RTN, rht_group=0)
    qb = oracle.quantize(b, oracle.RTN, rht_group=0)
    C = torch.full((M, N + 5), float("nan"), dtype=dtype, device="cuda")[:, :N]
    amax = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    w = ws(qii.qii_gemm_workspace_bytes(M, N, K)) if use_ws else None
    if w is not None:
        w.fill_(0x7E)     # stale scale bytes (448) for the padded rows of the re-tiled copy
    qii.qii_gemm_nvfp4_amax(nv_to_dev(qa), nv_to_dev(qb), C, amax, w)
    torch.cuda.synchronize()
    ref, absum = oracle.gemm(qa, qb, with_abs=True)
    check(C.float().cpu().numpy().astype(np.float64), ref, absum, dtype == torch.bfloat16)
    assert amax.item() == C.float().abs().max().item()


def test_forward_pass_hands_its_abs_max_to_the_next_layer(oracle):
    """Two layers in a row: the first emits max|Y| from its GEMM, the second takes it as the abs-max
    of its input and skips that pass.  Its saved tensors must equal the oracle's quantization of the
    very bytes of Y."""
    T, d0, d1, d2 = 384, 256, 512, 128
    Xb, W1b, _ = synth.linear_layer_bf16(T, d0, d1, seed=5)
    W2b = synth.normal_bf16((d2, d1), 0.02, seed=9)
    X, W1, W2 = to_dev(Xb), to_dev(W1b), to_dev(W2b)
    for mode in (qii.RTN, qii.RTN_46):
        Y1 = torch.empty((T, d1), dtype=torch.bfloat16, device="cuda")
        Y2 = torch.empty((T, d2), dtype=torch.bfloat16, device="cuda")
        amax_y = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        Xq1, Wq1 = qii.NVFP4Tensor.empty(T, d0), qii.NVFP4Tensor.empty(d1, d0)
        Xq2, Wq2 = qii.NVFP4Tensor.empty(T, d1), qii.NVFP4Tensor.empty(d2, d1)
        qii.qii_linear_fwd_amax(X, W1, mode, Y1, amax_y, Xq1, Wq1, ws(qii.qii_linear_fwd_workspace_bytes(T, d0, d1)))
        qii.qii_linear_fwd_amax(Y1, W2, mode, Y2, None, Xq2, Wq2, ws(qii.qii_linear_fwd_workspace_bytes(T, d1, d2)),
                                amax_x=amax_y)
        torch.cuda.synchronize()
        assert amax_y.item() == Y1.float().abs().max().item()
        y1_bits = Y1.view(torch.int16).cpu().numpy().view(np.uint16)
        oXq2, oWq2 = oracle.linear_fwd(y1_bits, W2b, mode=mode)
        assert_nv_equal(Xq2, oXq2, f"second layer's saved input, mode {mode}")
        assert_nv_equal(Wq2, oWq2, f"second layer's saved weight, mode {mode}")
        ref, absum = oracle.gemm(oXq2, oWq2, with_abs=True)
        check(bf16_to_f64(Y2), ref, absum, True)
