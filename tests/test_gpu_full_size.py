"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: one
linear layer forward + backward with tokens 16384, d_in 2048, d_out 8192 (bf16 inputs with
outlier channels).  Saved forward tensors are compared byte for byte; the three GEMM outputs are
compared on sampled entries (plus one full row and one full column of Y) that the oracle
computes one by one from its own quantized operands."""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii
from paper_2601_22813_amd import synth

from gpu_util import assert_nv_equal, to_dev, ws

pytestmark = pytest.mark.gpu


def sample_pairs(M, N, count, rng):
    return rng.integers(0, M, count), rng.integers(0, N, count)


def check_samples(C, a, b, ms, ns, oracle, bf16, what):
    ref, absum = oracle.gemm_sampled(a, b, ms, ns)
    got = C[torch.from_numpy(ms).cuda(), torch.from_numpy(ns).cuda()].float().cpu().numpy().astype(np.float64)
    tol = 1e-5 * absum + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0) + 1e-30
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {len(ms)} samples off, e.g. ({ms[bad][0]},{ns[bad][0]}) gpu {got[bad][0]} ref {ref[bad][0]}"


def test_linear_layer_at_benchmark_size(oracle):
    T, d_in, d_out = 16384, 2048, 8192
    rng = np.random.default_rng(0)
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=2)
    X, W, E = to_dev(Xb), to_dev(Wb), to_dev(Eb)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    print("forward", flush=True)
    qii.qii_linear_fwd(X, W, Y, Xq, Wq, ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out)))
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    assert_nv_equal(Xq, oXq, "saved X")
    assert_nv_equal(Wq, oWq, "saved W")
    ms, ns = sample_pairs(T, d_out, 4096, rng)
    ms = np.concatenate([ms, np.full(d_out, 12345), np.arange(T)])          # one full row
    ns = np.concatenate([ns, np.arange(d_out), np.full(T, 4321)])           # one full column
    check_samples(Y, oXq, oWq, ms, ns, oracle, True, "Y")
    print("backward", flush=True)
    dX = torch.empty((T, d_in), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device="cuda")
    seed = 2024
    qii.qii_linear_bwd(E, Xq, Wq, seed, dX, dW, ws(qii.qii_linear_bwd_workspace_bytes(T, d_in, d_out)))
    torch.cuda.synchronize()
    print("oracle operands", flush=True)
    Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, oXq, oWq, seed)
    ms, ns = sample_pairs(T, d_in, 4096, rng)
    check_samples(dX, Eq, WTq, ms, ns, oracle, True, "dX")
    ms, ns = sample_pairs(d_out, d_in, 4096, rng)
    check_samples(dW, ETq, XTq, ms, ns, oracle, True, "dW")
    # the quantized backward operands themselves, through the public quantizer with the derived seeds
    s = [qii.qii_derive_seed(seed, i) for i in range(6)]
    out = qii.NVFP4Tensor.empty(d_out, T)
    qii.qii_quantize_nvfp4(E, True, qii.MS_EDEN, 128, s[1], s[4], None, out, ws(256))
    assert_nv_equal(out, ETq, "Q(E^T)")
    out = qii.NVFP4Tensor.empty(d_in, T)
    qii.qii_requantize_nvfp4(Xq, True, qii.MS_EDEN, 128, s[1], s[5], None, out, ws(256))
    assert_nv_equal(out, XTq, "Q(X^T)")
    out = qii.NVFP4Tensor.empty(T, d_out)
    qii.qii_quantize_nvfp4(E, False, qii.MS_EDEN, 128, s[0], s[2], None, out, ws(256))
    assert_nv_equal(out, Eq, "Q(E)")


def test_paper_recipe_layer_at_benchmark_size(oracle):
    """The same layer as the paper runs it and as bench.py also times it: 4/6 on the forward pass
    (Sec. 4.1), post hoc range alignment on the backward pass (Sec. 7)."""
    T, d_in, d_out = 16384, 2048, 8192
    rng = np.random.default_rng(1)
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=2)
    X, W, E = to_dev(Xb), to_dev(Wb), to_dev(Eb)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    print("forward 4/6", flush=True)
    qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y, Xq, Wq, ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out)))
    oXq, oWq = oracle.linear_fwd(Xb, Wb, mode=oracle.RTN_46)
    assert_nv_equal(Xq, oXq, "saved X (4/6)")
    assert_nv_equal(Wq, oWq, "saved W (4/6)")
    ms, ns = sample_pairs(T, d_out, 4096, rng)
    check_samples(Y, oXq, oWq, ms, ns, oracle, True, "Y (4/6)")
    print("backward post hoc", flush=True)
    dX = torch.empty((T, d_in), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device="cuda")
    seed = 77
    qii.qii_linear_bwd_mode(E, Xq, Wq, seed, qii.MS_EDEN_PH, dX, dW,
                            ws(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH)))
    torch.cuda.synchronize()
    print("oracle operands", flush=True)
    Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, oXq, oWq, seed, mode=oracle.MS_EDEN_PH)
    ms, ns = sample_pairs(T, d_in, 4096, rng)
    check_samples(dX, Eq, WTq, ms, ns, oracle, True, "dX (post hoc)")
    ms, ns = sample_pairs(d_out, d_in, 4096, rng)
    check_samples(dW, ETq, XTq, ms, ns, oracle, True, "dW (post hoc)")
    # the four quantized operands, byte for byte, through the public quantizer with the derived seeds
    s = [qii.qii_derive_seed(seed, i) for i in range(6)]
    w = ws(qii.qii_quantize_posthoc_workspace_bytes(T, d_out))
    out = qii.NVFP4Tensor.empty(T, d_out)
    qii.qii_quantize_nvfp4(E, False, qii.MS_EDEN_PH, 128, s[0], s[2], None, out, w)
    assert_nv_equal(out, Eq, "Q(E) post hoc")
    out = qii.NVFP4Tensor.empty(d_out, T)
    qii.qii_quantize_nvfp4(E, True, qii.MS_EDEN_PH, 128, s[1], s[4], None, out, w)
    assert_nv_equal(out, ETq, "Q(E^T) post hoc")
    out = qii.NVFP4Tensor.empty(d_in, d_out)
    qii.qii_requantize_nvfp4(Wq, True, qii.MS_EDEN_PH, 128, s[0], s[3], None, out, w)
    assert_nv_equal(out, WTq, "Q(W^T) post hoc")
    out = qii.NVFP4Tensor.empty(d_in, T)
    qii.qii_requantize_nvfp4(Xq, True, qii.MS_EDEN_PH, 128, s[1], s[5], None, out, w)
    assert_nv_equal(out, XTq, "Q(X^T) post hoc")


# Larger workloads: the per-layer linears of the 1.9B decoder at T = 32768 tokens, the two
# roofline-stress shapes, and the 7B rows of the paper's table of Llama-like layer shapes (App. D)
# at 8 x 2048 tokens.  Shapes whose tile counts are not multiples of 8 (22016 / 256 = 86,
# 11008 / 256 = 43, 28672 / 256 = 112) also reach the tile walk without the XCD re-mapping and its
# remainder group.
LARGE_SHAPES = [
    ("decoder-1.9B down, T=32768", 32768, 8192, 2048, "paper"),
    ("decoder-1.9B qkv, T=32768", 32768, 2048, 6144, "plain"),
    ("stress 16384^3", 16384, 16384, 16384, "paper"),
    ("stress 16384x8192->28672", 16384, 8192, 28672, "plain"),
    ("7B UpGate", 16384, 4096, 22016, "paper"),
    ("7B Down", 16384, 11008, 4096, "paper"),
]


@pytest.mark.parametrize("name,T,d_in,d_out,recipe", LARGE_SHAPES, ids=[s[0] for s in LARGE_SHAPES])
def test_layer_sampled_parity_at_large_shapes(oracle, name, T, d_in, d_out, recipe):
    """Saved forward tensors byte for byte; Y, dX and dW on 4096 sampled entries each, against the
    oracle's exact definition on its own quantized operands.  recipe "plain": RTN forward and
    Algorithm 1 backward; "paper": 4/6 forward and post hoc range alignment backward."""
    rng = np.random.default_rng(T + d_in + d_out)
    fwd_mode, bwd_mode = (qii.RTN_46, qii.MS_EDEN_PH) if recipe == "paper" else (qii.RTN, qii.MS_EDEN)
    print(f"{name}: inputs", flush=True)
    Xb, Wb, Eb = synth.linear_layer_bf16(T, d_in, d_out, seed=3)
    X, W, E = to_dev(Xb), to_dev(Wb), to_dev(Eb)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, d_in), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device="cuda")
    seed = 99
    print(f"{name}: forward + backward on the GPU", flush=True)
    qii.qii_linear_fwd_mode(X, W, fwd_mode, Y, Xq, Wq, ws(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out)))
    qii.qii_linear_bwd_mode(E, Xq, Wq, seed, bwd_mode, dX, dW,
                            ws(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, bwd_mode)))
    torch.cuda.synchronize()
    print(f"{name}: oracle forward", flush=True)
    oXq, oWq = oracle.linear_fwd(Xb, Wb, mode=fwd_mode)
    assert_nv_equal(Xq, oXq, f"{name}: saved X")
    assert_nv_equal(Wq, oWq, f"{name}: saved W")
    ms, ns = sample_pairs(T, d_out, 4096, rng)
    check_samples(Y, oXq, oWq, ms, ns, oracle, True, f"{name}: Y")
    print(f"{name}: oracle backward operands", flush=True)
    Eq, WTq, ETq, XTq = oracle.linear_bwd_operands(Eb, oXq, oWq, seed, mode=bwd_mode)
    ms, ns = sample_pairs(T, d_in, 4096, rng)
    check_samples(dX, Eq, WTq, ms, ns, oracle, True, f"{name}: dX")
    ms, ns = sample_pairs(d_out, d_in, 4096, rng)
    check_samples(dW, ETq, XTq, ms, ns, oracle, True, f"{name}: dW")
