"""CPU oracle of the NVFP4 linear-layer path (test infrastructure only).

Thin ctypes marshalling around ``qii_oracle.c`` plus the layer compositions of
Sec. 5 of the paper (forward pass / backward pass), which are pure call
sequences.  Nothing in the HIP library or its Python binding imports this
package; only tests, the smoke check and the benchmark's cpu_baseline leg do.

bf16 tensors are numpy ``uint16`` arrays holding the bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qii_oracle.c")
_LIB = os.path.join(_HERE, "libqii_oracle.so")

RTN, SR, MS_EDEN, RTN_46, MS_EDEN_PH = 0, 1, 2, 3, 4
F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict binary32: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        c = ctypes
        u8p, f32p, f64p, i64p = (c.POINTER(c.c_uint8), c.POINTER(c.c_float),
                                 c.POINTER(c.c_double), c.POINTER(c.c_int64))
        _lib.qo_philox4x32_10.argtypes = [c.POINTER(c.c_uint32)] * 3
        _lib.qo_philox4x32_10.restype = None
        _lib.qo_rht_signs.argtypes = [c.c_uint64, c.POINTER(c.c_uint32)]
        _lib.qo_rht_signs.restype = None
        _lib.qo_scale_draw.argtypes = [c.c_uint64, c.c_int64, c.c_int64]
        _lib.qo_scale_draw.restype = c.c_uint32
        _lib.qo_elem_draw.argtypes = [c.c_uint64, c.c_int64, c.c_int64]
        _lib.qo_elem_draw.restype = c.c_uint32
        _lib.qo_derive_seed.argtypes = [c.c_uint64, c.c_uint32]
        _lib.qo_derive_seed.restype = c.c_uint64
        _lib.qo_e2m1_decode.argtypes = [c.c_uint8]
        _lib.qo_e2m1_decode.restype = c.c_float
        _lib.qo_e2m1_rtn.argtypes = [c.c_float]
        _lib.qo_e2m1_rtn.restype = c.c_uint8
        _lib.qo_e2m1_sr.argtypes = [c.c_float, c.c_uint32]
        _lib.qo_e2m1_sr.restype = c.c_uint8
        _lib.qo_e4m3_decode.argtypes = [c.c_uint8]
        _lib.qo_e4m3_decode.restype = c.c_float
        _lib.qo_e4m3_rtn.argtypes = [c.c_float]
        _lib.qo_e4m3_rtn.restype = c.c_uint8
        _lib.qo_e8m3_rtn.argtypes = [c.c_float]
        _lib.qo_e8m3_rtn.restype = c.c_float
        _lib.qo_e4m3_sr.argtypes = [c.c_float, c.c_uint32]
        _lib.qo_e4m3_sr.restype = c.c_uint8
        _lib.qo_rht.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_int,
                                c.c_int, c.c_uint64, f32p, f32p]
        _lib.qo_rht.restype = c.c_int
        _lib.qo_quantize.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_int,
                                     c.c_int, c.c_int, c.c_uint64, c.c_uint64, f32p, c.c_float,
                                     u8p, u8p, f32p]
        _lib.qo_quantize.restype = c.c_int
        _lib.qo_dequantize.argtypes = [u8p, u8p, f32p, c.c_int64, c.c_int64, f32p]
        _lib.qo_dequantize.restype = c.c_int
        _lib.qo_requantize.argtypes = [u8p, u8p, f32p, c.c_int64, c.c_int64, c.c_int, c.c_int,
                                       c.c_int, c.c_uint64, c.c_uint64, f32p, u8p, u8p, f32p]
        _lib.qo_requantize.restype = c.c_int
        _lib.qo_gemm.argtypes = [u8p, u8p, f32p, c.c_int64, u8p, u8p, f32p, c.c_int64, c.c_int64,
                                 f64p, f64p]
        _lib.qo_gemm.restype = c.c_int
        _lib.qo_gemm_sampled.argtypes = [u8p, u8p, f32p, u8p, u8p, f32p, c.c_int64, i64p, i64p,
                                         c.c_int64, f64p, f64p]
        _lib.qo_gemm_sampled.restype = c.c_int
        _lib.qo_max_threads.argtypes = []
        _lib.qo_max_threads.restype = c.c_int
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments")


@dataclass
class NVFP4:
    """The triple {x^FP4, x^FP8, x^FP32} of Sec. 3.1 for a rows x cols tensor."""
    codes: np.ndarray         # uint8 [rows, cols // 2], element 2j in the low nibble
    scales: np.ndarray        # uint8 [rows, cols // 16], E4M3 bytes
    tensor_scale: np.ndarray  # float32 [1]

    @property
    def rows(self) -> int:
        return self.codes.shape[0]

    @property
    def cols(self) -> int:
        return self.codes.shape[1] * 2


def _dtype_of(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.uint16:
        return BF16
    raise TypeError("oracle inputs are float32, or uint16 holding bf16 bit patterns")


def max_threads() -> int:
    return int(lib().qo_max_threads())


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().qo_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def rht_signs(seed_rht: int) -> np.ndarray:
    """The 128 entries (+1 / -1) of the sign vector of omega_RHT."""
    w = np.zeros(4, dtype=np.uint32)
    lib().qo_rht_signs(ctypes.c_uint64(seed_rht), _p(w, ctypes.c_uint32))
    bits = np.array([(int(w[j >> 5]) >> (j & 31)) & 1 for j in range(128)])
    return np.where(bits == 1, -1.0, 1.0)


def scale_draw(seed_sr: int, row: int, cg: int) -> int:
    return int(lib().qo_scale_draw(ctypes.c_uint64(seed_sr), row, cg))


def elem_draw(seed_sr: int, row: int, col: int) -> int:
    return int(lib().qo_elem_draw(ctypes.c_uint64(seed_sr), row, col))


def derive_seed(seed: int, i: int) -> int:
    return int(lib().qo_derive_seed(ctypes.c_uint64(seed), i))


def e2m1_decode(code: int) -> float:
    return float(lib().qo_e2m1_decode(code))


def e2m1_rtn(q: float) -> int:
    return int(lib().qo_e2m1_rtn(ctypes.c_float(q)))


def e2m1_sr(q: float, r16: int) -> int:
    return int(lib().qo_e2m1_sr(ctypes.c_float(q), r16))


def e4m3_decode(b: int) -> float:
    return float(lib().qo_e4m3_decode(b))


def e4m3_rtn(r: float) -> int:
    return int(lib().qo_e4m3_rtn(ctypes.c_float(r)))


def e8m3_rtn(u: float) -> float:
    return float(lib().qo_e8m3_rtn(ctypes.c_float(u)))


def e4m3_sr(t: float, r20: int) -> int:
    return int(lib().qo_e4m3_sr(ctypes.c_float(t), r20))


def rht(x: np.ndarray, transpose: bool = False, rht_group: int = 128, seed_rht: int = 0):
    """Rotated (and possibly transposed) x as float32, and its absolute maximum."""
    x = np.ascontiguousarray(x)
    rows, cols = x.shape
    R, C = (cols, rows) if transpose else (rows, cols)
    y = np.zeros((R, C), dtype=np.float32)
    amax = np.zeros(1, dtype=np.float32)
    _check(lib().qo_rht(x.ctypes.data, _dtype_of(x), rows, cols, cols, int(transpose), rht_group,
                        ctypes.c_uint64(seed_rht), _p(y, ctypes.c_float), _p(amax, ctypes.c_float)),
           "rht")
    return y, float(amax[0])


def quantize(x: np.ndarray, mode: int, transpose: bool = False, rht_group: int = 128,
             seed_rht: int = 0, seed_sr: int = 0, amax: float | None = None,
             s_override: float = 0.0) -> NVFP4:
    """Q(x) (or Q(x^T)) with mode RTN | SR | MS_EDEN | RTN_46 | MS_EDEN_PH; output lives in rotated space."""
    x = np.ascontiguousarray(x)
    rows, cols = x.shape
    R, C = (cols, rows) if transpose else (rows, cols)
    if C % 16:
        raise ValueError("oracle: the quantized dimension must be a multiple of 16")
    out = NVFP4(np.zeros((R, C // 2), np.uint8), np.zeros((R, C // 16), np.uint8),
                np.zeros(1, np.float32))
    am = None
    if amax is not None:
        am_arr = np.array([amax], dtype=np.float32)
        am = _p(am_arr, ctypes.c_float)
    _check(lib().qo_quantize(x.ctypes.data, _dtype_of(x), rows, cols, cols, int(transpose), mode,
                             rht_group, ctypes.c_uint64(seed_rht), ctypes.c_uint64(seed_sr), am,
                             ctypes.c_float(s_override), _p(out.codes, ctypes.c_uint8),
                             _p(out.scales, ctypes.c_uint8), _p(out.tensor_scale, ctypes.c_float)),
           "quantize")
    return out


def dequantize(q: NVFP4) -> np.ndarray:
    y = np.zeros((q.rows, q.cols), dtype=np.float32)
    _check(lib().qo_dequantize(_p(q.codes, ctypes.c_uint8), _p(q.scales, ctypes.c_uint8),
                               _p(q.tensor_scale, ctypes.c_float), q.rows, q.cols,
                               _p(y, ctypes.c_float)), "dequantize")
    return y


def requantize(q: NVFP4, mode: int, transpose: bool = True, rht_group: int = 128,
               seed_rht: int = 0, seed_sr: int = 0, amax: float | None = None) -> NVFP4:
    """Dequantize a saved tensor, optionally transpose, quantize again (Sec. 5, backward)."""
    R, C = (q.cols, q.rows) if transpose else (q.rows, q.cols)
    out = NVFP4(np.zeros((R, C // 2), np.uint8), np.zeros((R, C // 16), np.uint8),
                np.zeros(1, np.float32))
    am = None
    if amax is not None:
        am_arr = np.array([amax], dtype=np.float32)
        am = _p(am_arr, ctypes.c_float)
    _check(lib().qo_requantize(_p(q.codes, ctypes.c_uint8), _p(q.scales, ctypes.c_uint8),
                               _p(q.tensor_scale, ctypes.c_float), q.rows, q.cols, int(transpose),
                               mode, rht_group, ctypes.c_uint64(seed_rht), ctypes.c_uint64(seed_sr),
                               am, _p(out.codes, ctypes.c_uint8), _p(out.scales, ctypes.c_uint8),
                               _p(out.tensor_scale, ctypes.c_float)), "requantize")
    return out


def gemm(a: NVFP4, b: NVFP4, with_abs: bool = False):
    """C = A_hat * B_hat^T in double (A is M x K, B is N x K)."""
    if a.cols != b.cols:
        raise ValueError("oracle: inner dimensions differ")
    M, N, K = a.rows, b.rows, a.cols
    C = np.zeros((M, N), dtype=np.float64)
    S = np.zeros((M, N), dtype=np.float64) if with_abs else None
    _check(lib().qo_gemm(_p(a.codes, ctypes.c_uint8), _p(a.scales, ctypes.c_uint8),
                         _p(a.tensor_scale, ctypes.c_float), M, _p(b.codes, ctypes.c_uint8),
                         _p(b.scales, ctypes.c_uint8), _p(b.tensor_scale, ctypes.c_float), N, K,
                         _p(C, ctypes.c_double), _p(S, ctypes.c_double) if with_abs else None),
           "gemm")
    return (C, S) if with_abs else C


def gemm_sampled(a: NVFP4, b: NVFP4, ms: np.ndarray, ns: np.ndarray):
    """The GEMM definition at the listed (m, n) pairs: values and sums of |products|."""
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    out = np.zeros(ms.shape[0], dtype=np.float64)
    absum = np.zeros(ms.shape[0], dtype=np.float64)
    _check(lib().qo_gemm_sampled(_p(a.codes, ctypes.c_uint8), _p(a.scales, ctypes.c_uint8),
                                 _p(a.tensor_scale, ctypes.c_float), _p(b.codes, ctypes.c_uint8),
                                 _p(b.scales, ctypes.c_uint8), _p(b.tensor_scale, ctypes.c_float),
                                 a.cols, _p(ms, ctypes.c_int64), _p(ns, ctypes.c_int64),
                                 ms.shape[0], _p(out, ctypes.c_double), _p(absum, ctypes.c_double)),
           "gemm_sampled")
    return out, absum


# Sub-seed indices of the backward pass (one layer seed -> two rotations, four roundings).
SEED_RHT_DGRAD, SEED_RHT_WGRAD, SEED_SR_E, SEED_SR_WT, SEED_SR_ET, SEED_SR_XT = range(6)


def linear_fwd(X: np.ndarray, W: np.ndarray, mode: int = RTN):
    """Sec. 5, forward pass: RTN-quantize X (T x d_in) and W (d_out x d_in) along d_in with the
    native 1x16 scales and no rotation, multiply, keep the quantized tensors; mode RTN_46 adds
    the per-block 4/6 choice of Sec. 4.1.
    Returns (Xq, Wq); Y = gemm(Xq, Wq) is left to the caller (it is O(T d_in d_out))."""
    Xq = quantize(X, mode, rht_group=0)
    Wq = quantize(W, mode, rht_group=0)
    return Xq, Wq


def linear_bwd_operands(E: np.ndarray, Xq: NVFP4, Wq: NVFP4, seed: int, mode: int = MS_EDEN):
    """Sec. 5, backward pass: the four MS-EDEN operands (mode MS_EDEN, or MS_EDEN_PH for the
    post hoc range alignment of Sec. 7).
    dX = gemm(Eq, WTq)  (inner dimension d_out, both rotated with sub-seed 0);
    dW = gemm(ETq, XTq) (inner dimension T,     both rotated with sub-seed 1)."""
    s = [derive_seed(seed, i) for i in range(6)]
    Eq = quantize(E, mode, seed_rht=s[SEED_RHT_DGRAD], seed_sr=s[SEED_SR_E])
    WTq = requantize(Wq, mode, transpose=True, seed_rht=s[SEED_RHT_DGRAD], seed_sr=s[SEED_SR_WT])
    ETq = quantize(E, mode, transpose=True, seed_rht=s[SEED_RHT_WGRAD], seed_sr=s[SEED_SR_ET])
    XTq = requantize(Xq, mode, transpose=True, seed_rht=s[SEED_RHT_WGRAD], seed_sr=s[SEED_SR_XT])
    return Eq, WTq, ETq, XTq
