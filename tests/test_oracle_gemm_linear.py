"""Pins of the oracle's block-scaled GEMM and of the layer compositions of Sec. 5:
a library matmul of independently dequantized operands, integer arithmetic for the
unit-scale case, and the statistical statement that the backward-pass products average
to the products of the forward-quantized tensors with the unquantized gradient."""
import numpy as np
import torch

from paper_2601_22813_amd import synth

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, -0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0])


def unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1)


def dequant_f64(q):
    s = torch.from_numpy(q.scales).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    return E2M1[unpack(q.codes)] * np.repeat(s, 16, axis=1) * float(q.tensor_scale[0])


def test_gemm_is_the_product_of_the_dequantized_operands(oracle):
    rng = np.random.default_rng(0)
    a = rng.standard_normal((24, 160)).astype(np.float32)
    b = (rng.standard_normal((40, 160)) * 0.02).astype(np.float32)
    qa = oracle.quantize(a, oracle.RTN, rht_group=0)
    qb = oracle.quantize(b, oracle.SR, rht_group=0, seed_sr=3)
    C, S = oracle.gemm(qa, qb, with_abs=True)
    A, B = dequant_f64(qa), dequant_f64(qb)
    assert C.shape == (24, 40)
    assert np.allclose(C, A @ B.T, rtol=1e-12, atol=1e-15)
    assert np.allclose(S, np.abs(A) @ np.abs(B).T, rtol=1e-12)
    # a transposed-operand mistake would show here: the product is not symmetric
    assert not np.allclose(C[:24, :24], C[:24, :24].T)
    ms = np.array([0, 5, 23, 7]); ns = np.array([0, 39, 11, 7])
    vals, sums = oracle.gemm_sampled(qa, qb, ms, ns)
    assert np.array_equal(vals, C[ms, ns]) and np.array_equal(sums, S[ms, ns])


def test_gemm_unit_scales_is_integer_arithmetic(oracle):
    # all scale bytes 0x38 (= 1.0) and tensor scale 1: products are multiples of 1/4
    rng = np.random.default_rng(1)
    M, N, K = 16, 8, 256
    ca = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    cb = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    one = np.ones(1, dtype=np.float32)
    qa = oracle.NVFP4(ca, np.full((M, K // 16), 0x38, np.uint8), one)
    qb = oracle.NVFP4(cb, np.full((N, K // 16), 0x38, np.uint8), one.copy())
    C = oracle.gemm(qa, qb)
    ia = np.rint(E2M1[unpack(ca)] * 2).astype(np.int64)
    ib = np.rint(E2M1[unpack(cb)] * 2).astype(np.int64)
    assert np.array_equal(C * 4, (ia @ ib.T).astype(np.float64))


def test_quantized_product_approximates_the_real_one(oracle):
    # both operands rotated with the same seed on the inner dimension: the product estimates
    # a b^T without any inverse rotation, with error set by the two quantization errors
    rng = np.random.default_rng(2)
    a = rng.standard_normal((64, 512)).astype(np.float32)
    b = rng.standard_normal((48, 512)).astype(np.float32)
    qa = oracle.quantize(a, oracle.MS_EDEN, seed_rht=4, seed_sr=5)
    qb = oracle.quantize(b, oracle.MS_EDEN, seed_rht=4, seed_sr=6)
    C = oracle.gemm(qa, qb)
    ref = a.astype(np.float64) @ b.astype(np.float64).T
    rel = ((C - ref) ** 2).sum() / (ref ** 2).sum()
    assert 0.01 < rel < 0.03        # about 2 x 9.4e-3 (Table 1)
    qb_other = oracle.quantize(b, oracle.MS_EDEN, seed_rht=99, seed_sr=6)
    bad = oracle.gemm(qa, qb_other)
    assert ((bad - ref) ** 2).sum() / (ref ** 2).sum() > 0.5   # mismatched rotations do not cancel


def test_linear_forward_and_backward_compositions(oracle):
    T, d_in, d_out = 256, 128, 384
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=5)
    X, W, E = (synth.bf16_bits_to_f32(t).astype(np.float64) for t in (Xb, Wb, Eb))
    Xq, Wq = oracle.linear_fwd(Xb, Wb)
    # forward: plain RTN with 1x16 scales along d_in, no rotation
    ref = oracle.quantize(synth.bf16_bits_to_f32(Xb), oracle.RTN, rht_group=0)
    assert np.array_equal(Xq.codes, ref.codes) and np.array_equal(Xq.scales, ref.scales)
    Y = oracle.gemm(Xq, Wq)
    assert Y.shape == (T, d_out)
    assert ((Y - X @ W.T) ** 2).sum() / ((X @ W.T) ** 2).sum() < 0.03
    Xh, Wh = dequant_f64(Xq), dequant_f64(Wq)
    dX_ref, dW_ref = E @ Wh, E.T @ Xh     # what the backward pass estimates
    B = 48
    accX, accW = np.zeros_like(dX_ref), np.zeros_like(dW_ref)
    e1x = e1w = 0.0
    for seed in range(B):
        Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, Xq, Wq, seed)
        assert (Eq.rows, Eq.cols) == (T, d_out) and (WTq.rows, WTq.cols) == (d_in, d_out)
        assert (ETq.rows, ETq.cols) == (d_out, T) and (XTq.rows, XTq.cols) == (d_in, T)
        dX, dW = oracle.gemm(Eq, WTq), oracle.gemm(ETq, XTq)
        accX += dX; accW += dW
        e1x += ((dX - dX_ref) ** 2).sum() / (dX_ref ** 2).sum() / B
        e1w += ((dW - dW_ref) ** 2).sum() / (dW_ref ** 2).sum() / B
    assert 0.005 < e1x < 0.04 and 0.005 < e1w < 0.04
    errX = ((accX / B - dX_ref) ** 2).sum() / (dX_ref ** 2).sum()
    errW = ((accW / B - dW_ref) ** 2).sum() / (dW_ref ** 2).sum()
    # unbiased: the error of the mean is the single-sample error divided by B
    assert errX * B / e1x < 1.6 and errW * B / e1w < 1.6
    # the six sub-seeds are distinct and the two GEMMs use different rotations
    seeds = [oracle.derive_seed(7, i) for i in range(6)]
    assert len(set(seeds)) == 6
    Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, Xq, Wq, 7)
    direct = oracle.quantize(Eb, oracle.MS_EDEN, seed_rht=seeds[0], seed_sr=seeds[2])
    assert np.array_equal(Eq.codes, direct.codes) and np.array_equal(Eq.scales, direct.scales)
    direct = oracle.requantize(Xq, oracle.MS_EDEN, transpose=True, seed_rht=seeds[1], seed_sr=seeds[5])
    assert np.array_equal(XTq.codes, direct.codes) and np.array_equal(XTq.scales, direct.scales)
