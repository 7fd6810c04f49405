"""Helpers of the GPU parity tests: numpy <-> device tensors, NVFP4 containers."""
import numpy as np
import torch

from paper_2601_22813_amd import binding as qii


def to_dev(x: np.ndarray) -> torch.Tensor:
    """float32 stays float32; uint16 is taken as bf16 bit patterns."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def nv_to_dev(q) -> qii.NVFP4Tensor:
    return qii.NVFP4Tensor(torch.from_numpy(q.codes).cuda(), torch.from_numpy(q.scales).cuda(),
                           torch.from_numpy(q.tensor_scale).cuda(), q.rows, q.cols)


def nv_bytes(t: qii.NVFP4Tensor):
    torch.cuda.synchronize()
    return t.codes.cpu().numpy(), t.scales.cpu().numpy(), t.tensor_scale.cpu().numpy()


def assert_nv_equal(t: qii.NVFP4Tensor, q, what=""):
    codes, scales, ts = nv_bytes(t)
    assert ts.view(np.uint32)[0] == q.tensor_scale.view(np.uint32)[0], f"{what}: tensor scale {ts} vs {q.tensor_scale}"
    bad_s = np.argwhere(scales != q.scales)
    assert bad_s.size == 0, f"{what}: {len(bad_s)} scale bytes differ, first at {bad_s[0]}: gpu {scales[tuple(bad_s[0])]} oracle {q.scales[tuple(bad_s[0])]}"
    bad_c = np.argwhere(codes != q.codes)
    assert bad_c.size == 0, f"{what}: {len(bad_c)} code bytes differ, first at {bad_c[0]}: gpu {codes[tuple(bad_c[0])]:#x} oracle {q.codes[tuple(bad_c[0])]:#x}"


def ws(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)
