"""The measurement aid qii_microbench: every kind runs on small inputs, and the kinds that move
data move exactly what their description says (so that the rates bench.py --microbench derives
from them count the right bytes)."""
import numpy as np
import pytest
import torch

from paper_2601_22813_amd import binding as qii

pytestmark = pytest.mark.gpu


def test_copy_write_and_traffic_kinds_touch_what_they_say():
    n = 1 << 20
    a = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    b = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
    qii.qii_microbench(qii.MB_COPY, a, b, n, 37, 0)          # a grid that does not divide the size
    torch.cuda.synchronize()
    assert torch.equal(b[:n], a) and int(b[n:].sum()) == 0
    b.zero_()
    qii.qii_microbench(qii.MB_WRITE, None, b, n, 5, 0)
    torch.cuda.synchronize()
    assert int((b[:n].view(torch.int32).view(-1, 4)[:, 2] != 3).sum()) == 0 and int(b[n:].sum()) == 0
    qii.qii_microbench(qii.MB_READ, a, b, n, 64, 0)
    # the quantizers' traffic patterns: every output byte of codes and scales is written once
    S = 8192
    x = torch.randint(1, 255, (S * S * 2,), dtype=torch.uint8, device="cuda")
    for kind, variants in ((qii.MB_QUANT_TRAFFIC, (0,)), (qii.MB_QUANT_TRAFFIC_COLS, (0, 1, 2, 3, 4, 5, 6))):
        for v in variants:
            out = torch.full((S * S // 2 + S * S // 16 + 256,), 0xA5, dtype=torch.uint8, device="cuda")
            qii.qii_microbench(kind, x, out, S * S * 2, 1, v)
            torch.cuda.synchronize()
            assert int((out[S * S // 2 + S * S // 16:] != 0xA5).sum()) == 0, (kind, v)     # nothing beyond the outputs
    torch.cuda.synchronize()


def test_issue_rate_and_atomic_kinds_run():
    b = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    for kind in (qii.MB_EMPTY, qii.MB_VALU_FMA, qii.MB_VALU_RHT, qii.MB_VALU_CVT_FP4, qii.MB_MFMA_F16,
                 qii.MB_VALU_CVT_F16_FP4, qii.MB_VALU_PK_MUL_F16, qii.MB_VALU_CVT_PK32_F16_FP6):
        qii.qii_microbench(kind, None, b, 0, 8, 4)
    for n in (0, 1, 2, 3, 4):
        qii.qii_microbench(qii.MB_MFMA_DEQUANT, None, b, n, 4, 2)
    qii.qii_microbench(qii.MB_ATOMIC_ONE_WORD, b, None, 0, 100, 0)
    torch.cuda.synchronize()
    assert int(b[:4].view(torch.int32)[0]) == 100            # the maximum of block index + 1
    b.zero_()
    qii.qii_microbench(qii.MB_ATOMIC_SPREAD, b, None, 0, 256, 0)
    torch.cuda.synchronize()
    words = b.view(torch.int32).view(64, 64)[:, 0].cpu().numpy()
    assert np.array_equal(words, np.arange(64) + 193)        # word w holds the largest block index + 1 with index % 64 == w
    with pytest.raises(qii.QiiError):
        qii.qii_microbench(99, None, None, 0, 1, 0)
