"""Thin ctypes binding of libqii (the C ABI declared in include/qii.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  torch is
used for device memory and the current stream, nothing else.  Importing works without
the built library; the first call raises if ``libqii.so`` is missing (there is no CPU
fallback).
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqii.so")

RTN, SR, MS_EDEN, RTN_46, MS_EDEN_PH = 0, 1, 2, 3, 4
F32, BF16 = 0, 1

EXPORTS = [
    "qii_rht", "qii_absmax", "qii_quantize_nvfp4", "qii_requantize_nvfp4", "qii_dequantize_nvfp4",
    "qii_gemm_nvfp4", "qii_linear_fwd", "qii_linear_fwd_mode", "qii_linear_bwd", "qii_linear_bwd_mode",
    "qii_quantize_workspace_bytes", "qii_quantize_posthoc_workspace_bytes", "qii_linear_bwd_mode_workspace_bytes",
    "qii_gemm_workspace_bytes", "qii_linear_fwd_workspace_bytes", "qii_linear_bwd_workspace_bytes",
    "qii_derive_seed", "qii_status_string", "qii_last_error", "qii_version", "qii_selftest_conversions", "qii_microbench", "qii_gemm_nvfp4_inexact", "qii_gemm_inexact_workspace_bytes",
    "qii_quantize_nvfp4_noalloc", "qii_gemm_nvfp4_amax", "qii_linear_fwd_amax",
    "qii_quantize_pair_nvfp4", "qii_quantize_pair_workspace_bytes",
    "qii_gemm_sharing_plan", "qii_gemm_sharing_segments", "qii_gemm_sharing_tile_slots",
]


class _NVFP4(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("tensor_scale", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64)]


class QiiError(RuntimeError):
    pass


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise QiiError(f"{LIB_PATH} is not built: run `python -m paper_2601_22813_amd.build` "
                           "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i64, u64, sz = c.c_void_p, c.c_int64, c.c_uint64, c.c_size_t
        nv = c.POINTER(_NVFP4)
        L.qii_rht.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, u64, vp, vp, vp]
        L.qii_absmax.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, c.c_int, u64, vp, vp]
        L.qii_quantize_nvfp4.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, c.c_int, c.c_int, u64,
                                         u64, vp, nv, vp, sz, vp]
        L.qii_quantize_nvfp4_noalloc.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, c.c_int, c.c_int, u64, u64, nv, vp]
        L.qii_quantize_nvfp4_noalloc.restype = c.c_int
        L.qii_quantize_pair_nvfp4.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, u64, u64, u64, u64, nv, nv, vp, sz, vp]
        L.qii_quantize_pair_nvfp4.restype = c.c_int
        L.qii_quantize_pair_workspace_bytes.argtypes = [i64, i64, c.c_int]
        L.qii_quantize_pair_workspace_bytes.restype = sz
        L.qii_requantize_nvfp4.argtypes = [nv, c.c_int, c.c_int, c.c_int, u64, u64, vp, nv, vp, sz, vp]
        L.qii_dequantize_nvfp4.argtypes = [nv, vp, vp]
        L.qii_gemm_nvfp4.argtypes = [nv, nv, vp, c.c_int, i64, vp, sz, vp]
        L.qii_gemm_nvfp4_amax.argtypes = [nv, nv, vp, c.c_int, i64, vp, vp, sz, vp]
        L.qii_gemm_nvfp4_inexact.argtypes = [nv, nv, vp, c.c_int, i64, c.c_int, vp, sz, vp]
        L.qii_gemm_nvfp4_inexact.restype = c.c_int
        L.qii_gemm_inexact_workspace_bytes.argtypes = [i64, i64, i64, c.c_int]
        L.qii_gemm_inexact_workspace_bytes.restype = sz
        L.qii_gemm_nvfp4_amax.restype = c.c_int
        L.qii_linear_fwd_amax.argtypes = [vp, vp, c.c_int, i64, i64, i64, c.c_int, vp, vp, vp, c.c_int, vp, nv, nv, vp, sz, vp]
        L.qii_linear_fwd_amax.restype = c.c_int
        L.qii_linear_fwd.argtypes = [vp, vp, c.c_int, i64, i64, i64, vp, c.c_int, nv, nv, vp, sz, vp]
        L.qii_linear_fwd_mode.argtypes = [vp, vp, c.c_int, i64, i64, i64, c.c_int, vp, vp, vp, c.c_int, nv, nv, vp, sz, vp]
        L.qii_linear_bwd.argtypes = [vp, c.c_int, nv, nv, u64, vp, vp, c.c_int, vp, sz, vp]
        L.qii_linear_bwd_mode.argtypes = [vp, c.c_int, nv, nv, u64, c.c_int, vp, vp, c.c_int, vp, sz, vp]
        L.qii_linear_bwd_mode.restype = c.c_int
        L.qii_quantize_posthoc_workspace_bytes.argtypes = [i64, i64]
        L.qii_quantize_posthoc_workspace_bytes.restype = sz
        L.qii_linear_bwd_mode_workspace_bytes.argtypes = [i64, i64, i64, c.c_int]
        L.qii_linear_bwd_mode_workspace_bytes.restype = sz
        for name in ("qii_rht", "qii_absmax", "qii_quantize_nvfp4", "qii_requantize_nvfp4",
                     "qii_dequantize_nvfp4", "qii_gemm_nvfp4", "qii_linear_fwd", "qii_linear_fwd_mode",
                     "qii_linear_bwd"):
            getattr(L, name).restype = c.c_int
        L.qii_quantize_workspace_bytes.argtypes = []
        L.qii_quantize_workspace_bytes.restype = sz
        for name in ("qii_gemm_workspace_bytes", "qii_linear_fwd_workspace_bytes",
                     "qii_linear_bwd_workspace_bytes"):
            getattr(L, name).argtypes = [i64, i64, i64]
            getattr(L, name).restype = sz
        L.qii_selftest_conversions.argtypes = [vp, vp]
        L.qii_selftest_conversions.restype = c.c_int
        L.qii_microbench.argtypes = [c.c_int, vp, vp, c.c_uint64, c.c_int, c.c_int, vp]
        L.qii_microbench.restype = c.c_int
        L.qii_derive_seed.argtypes = [u64, c.c_uint32]
        L.qii_derive_seed.restype = u64
        L.qii_status_string.argtypes = [c.c_int]
        L.qii_status_string.restype = c.c_char_p
        L.qii_last_error.argtypes = []
        L.qii_last_error.restype = c.c_char_p
        L.qii_version.argtypes = []
        L.qii_version.restype = c.c_int
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        L = lib()
        raise QiiError(f"{L.qii_status_string(status).decode()}: {L.qii_last_error().decode()}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _contig(*tensors):
    """The layer passes and GEMM outputs take dense row-major buffers: refuse a view whose rows
    are not contiguous instead of reading it with the wrong stride."""
    for t in tensors:
        if not t.is_contiguous():
            raise QiiError("this call takes contiguous tensors (got strides %s)" % (tuple(t.stride()),))


def _rows_contig(t):
    if t.dim() != 2 or t.stride(1) != 1:
        raise QiiError("this call takes a 2-D tensor with unit column stride (got strides %s)" % (tuple(t.stride()),))


@dataclass
class NVFP4Tensor:
    """Device buffers of one NVFP4 tensor (caller-owned, see qii_nvfp4 in include/qii.h)."""
    codes: torch.Tensor         # uint8 [rows, cols // 2]
    scales: torch.Tensor        # uint8 [rows, cols // 16]
    tensor_scale: torch.Tensor  # float32 [1]
    rows: int
    cols: int

    @staticmethod
    def empty(rows: int, cols: int, device="cuda") -> "NVFP4Tensor":
        return NVFP4Tensor(torch.empty((rows, cols // 2), dtype=torch.uint8, device=device),
                           torch.empty((rows, cols // 16), dtype=torch.uint8, device=device),
                           torch.empty(1, dtype=torch.float32, device=device), rows, cols)

    def c_struct(self) -> _NVFP4:
        return _NVFP4(self.codes.data_ptr(), self.scales.data_ptr(), self.tensor_scale.data_ptr(),
                      self.rows, self.cols)


def qii_version() -> int:
    return lib().qii_version()


def qii_derive_seed(seed: int, i: int) -> int:
    return int(lib().qii_derive_seed(seed, i))


def qii_quantize_workspace_bytes() -> int:
    return int(lib().qii_quantize_workspace_bytes())


def qii_linear_fwd_workspace_bytes(T: int, d_in: int, d_out: int) -> int:
    return int(lib().qii_linear_fwd_workspace_bytes(T, d_in, d_out))


def qii_quantize_posthoc_workspace_bytes(rows: int, cols: int) -> int:
    return int(lib().qii_quantize_posthoc_workspace_bytes(rows, cols))


def qii_linear_bwd_mode_workspace_bytes(T: int, d_in: int, d_out: int, mode: int) -> int:
    return int(lib().qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, mode))


def qii_linear_bwd_workspace_bytes(T: int, d_in: int, d_out: int) -> int:
    return int(lib().qii_linear_bwd_workspace_bytes(T, d_in, d_out))


def qii_selftest_conversions(counts: torch.Tensor):
    """counts: 8 x int64 on the device; receives the mismatch counts (see include/qii.h)."""
    _check(lib().qii_selftest_conversions(counts.data_ptr(), _stream()))


MB_EMPTY, MB_COPY, MB_READ, MB_WRITE, MB_QUANT_TRAFFIC, MB_VALU_FMA, MB_VALU_RHT, MB_VALU_CVT_FP4, MB_MFMA_F16, \
    MB_ATOMIC_ONE_WORD, MB_ATOMIC_SPREAD, MB_QUANT_TRAFFIC_COLS, MB_VALU_CVT_F16_FP4, \
    MB_VALU_PK_MUL_F16, MB_MFMA_DEQUANT, MB_VALU_CVT_PK32_F16_FP6 = range(16)


def qii_microbench(kind: int, a: torch.Tensor | None, b: torch.Tensor | None, n: int, blocks: int, iters: int):
    """One launch of a machine-limit microbenchmark (see include/qii.h); a, b: device byte buffers or None."""
    _check(lib().qii_microbench(kind, a.data_ptr() if a is not None else None, b.data_ptr() if b is not None else None,
                                n, blocks, iters, _stream()))


def qii_rht(x: torch.Tensor, transpose: bool, seed_rht: int, y: torch.Tensor, amax: torch.Tensor | None):
    _rows_contig(x)
    _contig(y)
    rows, cols = x.shape
    _check(lib().qii_rht(x.data_ptr(), _dt(x), rows, cols, x.stride(0), int(transpose), seed_rht,
                         y.data_ptr(), _ptr(amax), _stream()))


def qii_absmax(x: torch.Tensor, transpose: bool, rht_group: int, seed_rht: int, amax: torch.Tensor):
    _rows_contig(x)
    rows, cols = x.shape
    _check(lib().qii_absmax(x.data_ptr(), _dt(x), rows, cols, x.stride(0), int(transpose), rht_group,
                            seed_rht, amax.data_ptr(), _stream()))


def qii_quantize_nvfp4(x: torch.Tensor, transpose: bool, mode: int, rht_group: int, seed_rht: int,
                       seed_sr: int, amax_in: torch.Tensor | None, out: NVFP4Tensor,
                       ws: torch.Tensor | None):
    _rows_contig(x)
    rows, cols = x.shape
    s = out.c_struct()
    _check(lib().qii_quantize_nvfp4(x.data_ptr(), _dt(x), rows, cols, x.stride(0), int(transpose), mode,
                                    rht_group, seed_rht, seed_sr, _ptr(amax_in), ctypes.byref(s),
                                    _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                    _stream()))


def qii_quantize_nvfp4_noalloc(x: torch.Tensor, transpose: bool, mode: int, rht_group: int, seed_rht: int,
                               seed_sr: int, out: NVFP4Tensor):
    _rows_contig(x)
    rows, cols = x.shape
    s = out.c_struct()
    _check(lib().qii_quantize_nvfp4_noalloc(x.data_ptr(), _dt(x), rows, cols, x.stride(0), int(transpose), mode,
                                            rht_group, seed_rht, seed_sr, ctypes.byref(s), _stream()))


def qii_quantize_pair_workspace_bytes(rows: int, cols: int, mode: int) -> int:
    return int(lib().qii_quantize_pair_workspace_bytes(rows, cols, mode))


def qii_quantize_pair_nvfp4(x: torch.Tensor, mode: int, seed_rht_rows: int, seed_sr_rows: int, seed_rht_cols: int,
                            seed_sr_cols: int, out_rows: NVFP4Tensor, out_cols: NVFP4Tensor, ws: torch.Tensor):
    _rows_contig(x)
    rows, cols = x.shape
    sr, sc = out_rows.c_struct(), out_cols.c_struct()
    _check(lib().qii_quantize_pair_nvfp4(x.data_ptr(), _dt(x), rows, cols, x.stride(0), mode, seed_rht_rows, seed_sr_rows,
                                         seed_rht_cols, seed_sr_cols, ctypes.byref(sr), ctypes.byref(sc), ws.data_ptr(),
                                         ws.numel() * ws.element_size(), _stream()))


def qii_requantize_nvfp4(inp: NVFP4Tensor, transpose: bool, mode: int, rht_group: int, seed_rht: int,
                         seed_sr: int, amax_in: torch.Tensor | None, out: NVFP4Tensor,
                         ws: torch.Tensor | None):
    si, so = inp.c_struct(), out.c_struct()
    _check(lib().qii_requantize_nvfp4(ctypes.byref(si), int(transpose), mode, rht_group, seed_rht,
                                      seed_sr, _ptr(amax_in), ctypes.byref(so), _ptr(ws),
                                      0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def qii_dequantize_nvfp4(inp: NVFP4Tensor, y: torch.Tensor):
    si = inp.c_struct()
    _check(lib().qii_dequantize_nvfp4(ctypes.byref(si), y.data_ptr(), _stream()))


def qii_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().qii_gemm_workspace_bytes(M, N, K))


def qii_gemm_nvfp4(A: NVFP4Tensor, B: NVFP4Tensor, C: torch.Tensor, ws: torch.Tensor | None = None):
    _rows_contig(C)
    sa, sb = A.c_struct(), B.c_struct()
    _check(lib().qii_gemm_nvfp4(ctypes.byref(sa), ctypes.byref(sb), C.data_ptr(), _dt(C), C.stride(0),
                                _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream()))


INEXACT_FP8, INEXACT_FP4_POW2 = 0, 1


def qii_gemm_inexact_workspace_bytes(M: int, N: int, K: int, variant: int) -> int:
    return int(lib().qii_gemm_inexact_workspace_bytes(M, N, K, variant))


def qii_gemm_nvfp4_inexact(A: NVFP4Tensor, B: NVFP4Tensor, C: torch.Tensor, variant: int, ws: torch.Tensor):
    """Exploratory non-exact variants of the GEMM (measurement only; see include/qii.h)."""
    _rows_contig(C)
    sa, sb = A.c_struct(), B.c_struct()
    _check(lib().qii_gemm_nvfp4_inexact(ctypes.byref(sa), ctypes.byref(sb), C.data_ptr(), _dt(C), C.stride(0), variant,
                                        _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def qii_gemm_nvfp4_amax(A: NVFP4Tensor, B: NVFP4Tensor, C: torch.Tensor, amax_c: torch.Tensor | None,
                        ws: torch.Tensor | None = None):
    _rows_contig(C)
    sa, sb = A.c_struct(), B.c_struct()
    _check(lib().qii_gemm_nvfp4_amax(ctypes.byref(sa), ctypes.byref(sb), C.data_ptr(), _dt(C), C.stride(0),
                                     _ptr(amax_c), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                     _stream()))


def qii_linear_fwd_amax(X: torch.Tensor, W: torch.Tensor, mode: int, Y: torch.Tensor, amax_y: torch.Tensor | None,
                        Xq: NVFP4Tensor, Wq: NVFP4Tensor, ws: torch.Tensor, amax_x: torch.Tensor | None = None,
                        amax_w: torch.Tensor | None = None):
    _contig(X, W, Y)
    T, d_in = X.shape
    d_out = W.shape[0]
    sx, sw = Xq.c_struct(), Wq.c_struct()
    _check(lib().qii_linear_fwd_amax(X.data_ptr(), W.data_ptr(), _dt(X), T, d_in, d_out, mode, _ptr(amax_x),
                                     _ptr(amax_w), Y.data_ptr(), _dt(Y), _ptr(amax_y), ctypes.byref(sx),
                                     ctypes.byref(sw), ws.data_ptr(), ws.numel() * ws.element_size(), _stream()))


def qii_linear_fwd(X: torch.Tensor, W: torch.Tensor, Y: torch.Tensor, Xq: NVFP4Tensor,
                   Wq: NVFP4Tensor, ws: torch.Tensor):
    _contig(X, W, Y)
    T, d_in = X.shape
    d_out = W.shape[0]
    sx, sw = Xq.c_struct(), Wq.c_struct()
    _check(lib().qii_linear_fwd(X.data_ptr(), W.data_ptr(), _dt(X), T, d_in, d_out, Y.data_ptr(), _dt(Y),
                                ctypes.byref(sx), ctypes.byref(sw), ws.data_ptr(),
                                ws.numel() * ws.element_size(), _stream()))


def qii_linear_fwd_mode(X: torch.Tensor, W: torch.Tensor, mode: int, Y: torch.Tensor, Xq: NVFP4Tensor,
                        Wq: NVFP4Tensor, ws: torch.Tensor, amax_x: torch.Tensor | None = None,
                        amax_w: torch.Tensor | None = None):
    _contig(X, W, Y)
    T, d_in = X.shape
    d_out = W.shape[0]
    sx, sw = Xq.c_struct(), Wq.c_struct()
    _check(lib().qii_linear_fwd_mode(X.data_ptr(), W.data_ptr(), _dt(X), T, d_in, d_out, mode, _ptr(amax_x),
                                     _ptr(amax_w), Y.data_ptr(), _dt(Y), ctypes.byref(sx), ctypes.byref(sw),
                                     ws.data_ptr(), ws.numel() * ws.element_size(), _stream()))


def qii_linear_bwd(dY: torch.Tensor, Xq: NVFP4Tensor, Wq: NVFP4Tensor, seed: int, dX: torch.Tensor,
                   dW: torch.Tensor, ws: torch.Tensor):
    _contig(dY, dX, dW)
    if dW.dtype != dX.dtype:
        raise QiiError("dX and dW must have the same dtype")
    sx, sw = Xq.c_struct(), Wq.c_struct()
    _check(lib().qii_linear_bwd(dY.data_ptr(), _dt(dY), ctypes.byref(sx), ctypes.byref(sw), seed,
                                dX.data_ptr(), dW.data_ptr(), _dt(dX), ws.data_ptr(),
                                ws.numel() * ws.element_size(), _stream()))


def qii_linear_bwd_mode(dY: torch.Tensor, Xq: NVFP4Tensor, Wq: NVFP4Tensor, seed: int, mode: int,
                        dX: torch.Tensor, dW: torch.Tensor, ws: torch.Tensor):
    _contig(dY, dX, dW)
    if dW.dtype != dX.dtype:
        raise QiiError("dX and dW must have the same dtype")
    sx, sw = Xq.c_struct(), Wq.c_struct()
    _check(lib().qii_linear_bwd_mode(dY.data_ptr(), _dt(dY), ctypes.byref(sx), ctypes.byref(sw), seed, mode,
                                     dX.data_ptr(), dW.data_ptr(), _dt(dX), ws.data_ptr(),
                                     ws.numel() * ws.element_size(), _stream()))
