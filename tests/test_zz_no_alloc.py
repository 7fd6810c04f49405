"""The entry point that allocates nothing (qii_quantize_nvfp4_noalloc, scratch held by the library
in device memory) against qii_quantize_nvfp4 with a caller-owned workspace: identical bytes, on two
calls in a row, the second on a smaller tensor (the shared scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii
from paper_2601_22813_amd import synth

from gpu_util import to_dev, ws

pytestmark = pytest.mark.gpu


def both(x_np, transpose, mode, seed_rht, seed_sr):
    x = to_dev(x_np)
    rows, cols = x_np.shape
    R, C = (cols, rows) if transpose else (rows, cols)
    a, b = qii.NVFP4Tensor.empty(R, C), qii.NVFP4Tensor.empty(R, C)
    for t in (a, b):
        t.codes.fill_(0xAB); t.scales.fill_(0xCD); t.tensor_scale.fill_(-1.0)
    qii.qii_quantize_nvfp4_noalloc(x, transpose, mode, 128, seed_rht, seed_sr, a)
    qii.qii_quantize_nvfp4(x, transpose, mode, 128, seed_rht, seed_sr, None, b,
                           ws(qii.qii_quantize_posthoc_workspace_bytes(R, C)))
    torch.cuda.synchronize()
    return a, b


@pytest.mark.parametrize("mode", [qii.MS_EDEN, qii.MS_EDEN_PH, qii.RTN_46])
def test_noalloc_matches_the_workspace_entry_point_twice_in_a_row(mode):
    big = synth.student_t_bf16((512, 1024), 3, 0.1, seed=41)
    small = synth.normal_bf16((128, 256), 1e-3, seed=42)          # smaller, and a much smaller maximum
    for transpose in (False, True):
        for x_np in (big, small):
            a, b = both(x_np, transpose, mode, 7, 8)
            assert torch.equal(a.tensor_scale, b.tensor_scale), f"tensor scale, mode {mode} transpose {transpose} shape {x_np.shape}"
            assert torch.equal(a.scales, b.scales), f"scale bytes, mode {mode} transpose {transpose} shape {x_np.shape}"
            assert torch.equal(a.codes, b.codes), f"codes, mode {mode} transpose {transpose} shape {x_np.shape}"


def test_noalloc_refuses_what_its_scratch_cannot_hold():
    x = torch.zeros((8192, 8192 + 128), dtype=torch.bfloat16, device="cuda")
    out = qii.NVFP4Tensor.empty(8192, 8192 + 128)
    with pytest.raises(qii.QiiError, match="QII_UNSUPPORTED"):
        qii.qii_quantize_nvfp4_noalloc(x, False, qii.MS_EDEN_PH, 128, 0, 0, out)
    # the other modes only use the abs-max slot and take any size
    out.codes.fill_(0xAB)
    qii.qii_quantize_nvfp4_noalloc(x, False, qii.MS_EDEN, 128, 0, 0, out)
    torch.cuda.synchronize()
    assert int(out.codes.max()) == 0 and float(out.tensor_scale[0]) == 1.0
