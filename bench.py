#!/usr/bin/env python3
"""Benchmark of the NVFP4 linear-layer hot path on one MI355X.

One step = one pass of the whole path over synthetic inputs already resident in HBM:
  A1. the MS-EDEN quantizer on the quantize-only configuration (8192 x 8192 bf16,
      0.1 * Student-t(3), rotation groups of 128), blocks along rows and then along columns,
      with the tensor's abs-max supplied (the paper's App. D assumption): one read of the
      input from buffers that are cold in the 256 MiB Infinity Cache (four launches of each);
  A2. the same two quantizations as the literal two kernels of Algorithm 1 (rotated abs-max
      pass, then the quantize pass re-reading the tensor);
  A3. the same without a supplied abs-max in the two-kernel form of Sec. 7 (post hoc range
      alignment: heavy pass + scales-only pass), and both orientations from one read;
  B.  one linear layer forward + backward (tokens 16384, d_in 2048 -> d_out 8192, bf16):
      six quantizations and three block-scaled GEMMs, as RTN + Algorithm 1 and as the paper's
      recipe (4/6 forward, post hoc backward).
`value` is the quantizer's GB/s over part A3 (the headline metric on the quantize-only configuration, run
the way the paper's layer runs it: nothing supplied, all kernels of the scheme counted); the
abs-max-supplied and two-pass figures and the layer's TFLOP/s are reported beside it.  Inputs
rotate over 768 MiB of distinct buffers so that the Infinity Cache does not serve them.
After the timed steps the larger configurations (T = 32768 decoder linears, the two stress
shapes, the paper's table of layer shapes) are timed once each and added to the same JSON line.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
BYTES_PER_ELEM_QUANT = 2 + 0.5 + 0.0625      # bf16 in, packed FP4 + E4M3 scale out
BYTES_PER_ELEM_ABSMAX = 2.0                  # bf16 in
ALU_FLOPS_PER_ELEM = 16.5                    # arithmetic the contract asks of MS-EDEN with RHT-128, per element
VALU_F32_PEAK_TFLOPS = 157.3
# post hoc scheme: bf16 in, FP4 + one f32 per group out; then that f32 in, E4M3 scale out
BYTES_PER_ELEM_POSTHOC = 2 + 0.5 + 0.25 + 0.25 + 0.0625
# HBM bytes of one launch of the roofline kernel at 8192 x 8192, from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by
# the same counters' reading of a 512 MiB device copy: the row of that kernel in profiles/quantize_8192x8192_hbm_traffic.txt
TRAFFIC_QUANT_ROWS_BYTES = 172_160_000   # (that row to five digits: repeated runs differ by a few KB)


# Weight shapes [d_in, d_out] of Llama-like models (App. D, table of linear shapes), 8 x 2048 tokens.
PAPER_SHAPES = {
    "800M": {"QKV": (2048, 6144), "Out": (2048, 2048), "UpGate": (2048, 11264), "Down": (5632, 2048)},
    "3B": {"QKV": (3072, 9216), "Out": (3072, 3072), "UpGate": (3072, 16384), "Down": (8192, 3072)},
    "7B": {"QKV": (4096, 12288), "Out": (4096, 4096), "UpGate": (4096, 22016), "Down": (11008, 4096)},
    "22B": {"QKV": (6144, 18432), "Out": (6144, 6144), "UpGate": (6144, 32768), "Down": (16384, 6144)},
}


# Larger configurations: per-layer linears of a ~1.9B decoder at 32768 tokens per step, and the two stress shapes.
LARGE_CONFIGS = {
    "C4_decoder_1.9B_T32768": {"tokens": 32768, "layers": {"QKV": (2048, 6144), "O": (2048, 2048), "GateUp": (2048, 16384), "Down": (8192, 2048)}},
    "C5_stress": {"tokens": 16384, "layers": {"square_16384": (16384, 16384), "rect_8192_to_28672": (8192, 28672)}},
}


def time_layer(torch, qii, dev, T, d_in, d_out, reps=3):
    """ms of one layer forward + backward in the paper's recipe (4/6 forward with max|X|, max|W| supplied, post hoc
    MS-EDEN backward, all quantizers included), mean over `reps` runs after one warm-up."""
    g = torch.Generator(device=dev).manual_seed(1)
    X = torch.randn((T, d_in), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    W = (0.02 * torch.randn((d_out, d_in), device=dev, dtype=torch.float32, generator=g)).to(torch.bfloat16)
    E = (1e-3 * torch.randn((T, d_out), device=dev, dtype=torch.float32, generator=g)).to(torch.bfloat16)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device=dev)
    dX = torch.empty((T, d_in), dtype=torch.bfloat16, device=dev)
    dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device=dev)
    ws_f = torch.empty(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH), dtype=torch.uint8, device=dev)
    ax = torch.zeros(1, dtype=torch.float32, device=dev)
    aw = torch.zeros(1, dtype=torch.float32, device=dev)
    qii.qii_absmax(X, False, 0, 0, ax)
    qii.qii_absmax(W, False, 0, 0, aw)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = []
    for i in range(reps + 1):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y, Xq, Wq, ws_f, amax_x=ax, amax_w=aw)
        e1.record()
        qii.qii_linear_bwd_mode(E, Xq, Wq, i, qii.MS_EDEN_PH, dX, dW, ws_b)
        e2.record()
        torch.cuda.synchronize()
        if i:
            out.append((e0.elapsed_time(e1), e1.elapsed_time(e2)))
    fwd = float(np.mean([o[0] for o in out]))
    bwd = float(np.mean([o[1] for o in out]))
    return fwd, bwd


def large_configs(torch, qii, dev):
    res = {}
    for name, cfg in LARGE_CONFIGS.items():
        T = cfg["tokens"]
        layers, tot, flop = {}, 0.0, 0.0
        for lname, (d_in, d_out) in cfg["layers"].items():
            fwd, bwd = time_layer(torch, qii, dev, T, d_in, d_out)
            f = 6.0 * T * d_in * d_out
            layers[lname] = {"d_in": d_in, "d_out": d_out, "fwd_ms": round(fwd, 4), "bwd_ms": round(bwd, 4),
                             "TFLOPs": round(f / ((fwd + bwd) * 1e-3) / 1e12, 1)}
            tot += fwd + bwd
            flop += f
        res[name] = {"tokens": T, "ms": round(tot, 4), "TFLOPs": round(flop / (tot * 1e-3) / 1e12, 1),
                     "frac_of_mfma_peak": round(flop / (tot * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4), "layers": layers}
    res["note"] = ("forward + backward per layer, 4/6 forward (max|X|, max|W| supplied) + post hoc MS-EDEN backward, all "
                   "quantizers included; TFLOP/s = 6 T d_in d_out / time")
    return res


def paper_shapes(torch, qii, synth, dev):
    """Latency of forward + backward per model size, summed over its four layer shapes (the
    aggregation of the paper's linear-layer speed-up figure), for the NVFP4 layer of this library
    and for three plain bf16 matmuls (Y, dX, dW) of the same shapes."""
    T = 8 * 2048
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    for model, layers in PAPER_SHAPES.items():
        tot_q, tot_b, flop = 0.0, 0.0, 0.0
        per_layer = {}
        for name, (d_in, d_out) in layers.items():
            g = torch.Generator(device=dev).manual_seed(1)
            X = torch.randn((T, d_in), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
            W = (0.02 * torch.randn((d_out, d_in), device=dev, dtype=torch.float32, generator=g)).to(torch.bfloat16)
            E = (1e-3 * torch.randn((T, d_out), device=dev, dtype=torch.float32, generator=g)).to(torch.bfloat16)
            Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
            Y = torch.empty((T, d_out), dtype=torch.bfloat16, device=dev)
            dX = torch.empty((T, d_in), dtype=torch.bfloat16, device=dev)
            dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device=dev)
            ws_f = torch.empty(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out), dtype=torch.uint8, device=dev)
            ws_b = torch.empty(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH),
                               dtype=torch.uint8, device=dev)

            ax = torch.zeros(1, dtype=torch.float32, device=dev)
            aw = torch.zeros(1, dtype=torch.float32, device=dev)
            qii.qii_absmax(X, False, 0, 0, ax)     # supplied maxima, as the paper's layer timings assume (App. D)
            qii.qii_absmax(W, False, 0, 0, aw)

            def nvfp4(i):
                qii.qii_linear_fwd_mode(X, W, qii.RTN_46, Y, Xq, Wq, ws_f, amax_x=ax, amax_w=aw)
                qii.qii_linear_bwd_mode(E, Xq, Wq, i, qii.MS_EDEN_PH, dX, dW, ws_b)

            def bf16(i):
                torch.matmul(X, W.t(), out=Y)
                torch.matmul(E, W, out=dX)
                torch.matmul(E.t(), X, out=dW)

            ms = []
            for fn in (nvfp4, bf16):
                for i in range(2):
                    fn(i)
                torch.cuda.synchronize()
                e0, e1 = ev(), ev()
                e0.record()
                for i in range(5):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1) / 5)
            per_layer[name] = {"d_in": d_in, "d_out": d_out, "nvfp4_ms": round(ms[0], 4), "bf16_ms": round(ms[1], 4)}
            tot_q += ms[0]
            tot_b += ms[1]
            flop += 6.0 * T * d_in * d_out
            del X, W, E, Xq, Wq, Y, dX, dW, ws_f, ws_b
        out[model] = {"nvfp4_ms": round(tot_q, 4), "bf16_ms": round(tot_b, 4),
                      "nvfp4_TFLOPs": round(flop / (tot_q * 1e-3) / 1e12, 1),
                      "bf16_TFLOPs": round(flop / (tot_b * 1e-3) / 1e12, 1),
                      "speedup_over_bf16": round(tot_b / tot_q, 3), "layers": per_layer}
    out["note"] = ("tokens 16384; NVFP4 = 4/6 forward (max|X|, max|W| supplied) + post hoc MS-EDEN backward incl. all quantizers; bf16 = three "
                   "torch.matmul calls (vendor GEMM), no quantization; on this GPU the NVFP4 products run on the f16 "
                   "matrix instruction, whose peak equals the bf16 peak, so no speed-up over bf16 is possible here")
    return out


def inexact_gemm(torch, qii, synth, dev, T, d_in, d_out):
    """The exploratory non-exact GEMM variants on the forward GEMM of the benchmark's layer: time including their
    operand re-encoding pre-pass, and distance from the exact kernel's f32 result (which the GPU tests hold to 1e-5
    of the oracle's definition).  Context for what the native block-scaled matrix instruction would give if NVFP4's
    numerics were given up; never part of `value` or of the layer figures."""
    X_np, W_np, _ = synth.linear_layer_bf16(T, d_in, d_out, seed=2)
    to_dev = lambda b: torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
    X, W = to_dev(X_np), to_dev(W_np)
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    ws = torch.empty(256, dtype=torch.uint8, device=dev)
    qii.qii_quantize_nvfp4(X, False, qii.RTN, 0, 0, 0, None, Xq, ws)
    qii.qii_quantize_nvfp4(W, False, qii.RTN, 0, 0, 0, None, Wq, ws)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        out = []
        for i in range(reps + 1):
            e0, e1 = ev(), ev()
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            if i:
                out.append(e0.elapsed_time(e1))
        return float(np.mean(out))

    flops = 2.0 * T * d_in * d_out
    C_ex = torch.empty((T, d_out), dtype=torch.float32, device=dev)
    C16 = torch.empty((T, d_out), dtype=torch.bfloat16, device=dev)
    gws = torch.empty(max(256, qii.qii_gemm_workspace_bytes(T, d_out, d_in)), dtype=torch.uint8, device=dev)
    qii.qii_gemm_nvfp4(Xq, Wq, C_ex, gws)
    ms = timed(lambda: qii.qii_gemm_nvfp4(Xq, Wq, C16, gws))
    res = {"shape": {"M": T, "N": d_out, "K": d_in},
           "exact": {"ms": round(ms, 4), "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1)},
           "note": "non-exact variants, measurement only (qii_gemm_nvfp4_inexact; a plain kernel of 8 waves per tile without "
                   "software pipelining): times are for bf16 output and include the pre-pass that re-encodes both operands; "
                   "errors are of the f32 output against the exact kernel's, relative to the root mean square of its entries"}
    rms = float(C_ex.double().pow(2).mean().sqrt())
    C = torch.empty_like(C_ex)
    for name, variant in (("fp8_e4m3_pow2_scale_per_32", qii.INEXACT_FP8), ("fp4_zero_padded_pow2_scales", qii.INEXACT_FP4_POW2)):
        w = torch.empty(max(256, qii.qii_gemm_inexact_workspace_bytes(T, d_out, d_in, variant)), dtype=torch.uint8, device=dev)
        ms = timed(lambda: qii.qii_gemm_nvfp4_inexact(Xq, Wq, C16, variant, w))
        qii.qii_gemm_nvfp4_inexact(Xq, Wq, C, variant, w)
        torch.cuda.synchronize()
        d = (C - C_ex).double()
        res[name] = {"ms": round(ms, 4), "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1),
                     "rms_error_over_rms": round(float(d.pow(2).mean().sqrt()) / rms, 5),
                     "max_error_over_rms": round(float(d.abs().max()) / rms, 4)}
        del w, d
    return res


def microbench(torch, qii, dev):
    """Machine limits behind the roofline arguments, each one launch of qii_microbench timed with events (mean of 5
    after 2 warm-ups): streaming rates, the quantizer's traffic pattern without arithmetic, issue rates, atomics."""
    MiB = 2 ** 20
    a = torch.empty(512 * MiB, dtype=torch.uint8, device=dev).random_(0, 255)
    b = torch.empty(512 * MiB, dtype=torch.uint8, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def t_ms(fn, reps=6, warm=2):
        # launches back to back with an event between them, one synchronization at the end: the way the benchmark's
        # steps are timed, so that the figures compare
        e = [ev() for _ in range(reps + 1)]
        for i in range(warm):
            fn(i)
        e[0].record()
        for i in range(reps):
            fn(warm + i)
            e[i + 1].record()
        torch.cuda.synchronize()
        return float(np.mean([e[i].elapsed_time(e[i + 1]) for i in range(reps)]))

    res = {"note": "512 MiB buffers (twice the Infinity Cache); GB/s counts bytes read plus bytes written; clock taken as 2.4 GHz"}
    n = 512 * MiB
    for name, kind, nbytes in (("copy", qii.MB_COPY, 2 * n), ("read", qii.MB_READ, n), ("write", qii.MB_WRITE, n)):
        res[name] = {}
        for blocks in (1024, 2048, 4096, 32768):
            ms = t_ms(lambda i: qii.qii_microbench(kind, a, b, n, blocks, 0))
            res[name][f"blocks_{blocks}"] = {"ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
    # the rows quantizer's loads and stores on 8192 x 8192 bf16, a different (cold) 128 MiB input per launch
    nq = 128 * MiB
    ms = t_ms(lambda i: qii.qii_microbench(qii.MB_QUANT_TRAFFIC, a[(i % 4) * nq:], b, nq, 1, 0), reps=8)
    res["quantizer_rows_traffic_8192x8192_bf16"] = {"ms": round(ms, 4), "bytes": int(nq * (1 + 0.25 + 1 / 32)),
                                               "GBps": round(nq * (1 + 0.25 + 1 / 32) / (ms * 1e-3) / 1e9, 1)}
    ms = t_ms(lambda i: qii.qii_microbench(qii.MB_QUANT_TRAFFIC, a, b, nq, 1, 0), reps=8)
    res["quantizer_rows_traffic_8192x8192_bf16_same_input"] = {"ms": round(ms, 4), "GBps": round(nq * (1 + 0.25 + 1 / 32) / (ms * 1e-3) / 1e9, 1)}
    for order, oname in ((0, "row_blocks_fastest"), (1, "die_stripes"), (2, "column_blocks_fastest"),
                         (3, "lines_of_128B_waves_stacked"), (4, "lines_of_128B_waves_side_by_side"),
                         (5, "lines_of_128B_but_contiguous_stores"), (6, "lines_of_128B_but_contiguous_loads")):
        ms = t_ms(lambda i: qii.qii_microbench(qii.MB_QUANT_TRAFFIC_COLS, a[(i % 4) * nq:], b, nq, 1, order), reps=8)
        res.setdefault("quantizer_cols_traffic_8192x8192_bf16", {})[oname] = {
            "ms": round(ms, 4), "GBps": round(nq * (1 + 0.25 + 1 / 32) / (ms * 1e-3) / 1e9, 1)}
    # streaming at the quantizer's size: 128 MiB read (cold), and 128 MiB read + 32 MiB written by the copy kernel's
    # access pattern cannot be had from one kernel, so the two are given separately
    ms = t_ms(lambda i: qii.qii_microbench(qii.MB_READ, a[(i % 4) * nq:], b, nq, 8192, 0), reps=8)
    res["read_128MiB_cold"] = {"ms": round(ms, 4), "GBps": round(nq / (ms * 1e-3) / 1e9, 1)}
    ms = t_ms(lambda i: qii.qii_microbench(qii.MB_WRITE, None, b[(i % 4) * nq:], 36 * MiB, 2304, 0), reps=8)
    res["write_36MiB"] = {"ms": round(ms, 4), "GBps": round(36 * MiB / (ms * 1e-3) / 1e9, 1)}
    # issue rates: 2048 blocks of 4 waves (8 waves per SIMD)
    blocks, iters = 2048, 4096
    waves = blocks * 4
    cu_clk = 256 * 2.4e9
    for name, kind, per_trip in (("v_fma_f32", qii.MB_VALU_FMA, 16), ("rht128_slice", qii.MB_VALU_RHT, 128),
                                 ("v_cvt_scalef32_pk_fp4_f32", qii.MB_VALU_CVT_FP4, 8),
                                 ("v_cvt_scalef32_pk_f16_fp4", qii.MB_VALU_CVT_F16_FP4, 8), ("v_pk_mul_f16", qii.MB_VALU_PK_MUL_F16, 16),
                                 ("v_cvt_scalef32_pk32_f16_fp6", qii.MB_VALU_CVT_PK32_F16_FP6, 2)):
        ms = t_ms(lambda i: qii.qii_microbench(kind, None, b, 0, blocks, iters))
        wave_instr = waves * iters * per_trip
        res[name] = {"ms": round(ms, 4), "wave_instructions_per_CU_per_clock": round(wave_instr / (ms * 1e-3) / cu_clk, 3)}
    res["v_fma_f32"]["TFLOPs"] = round(waves * iters * 16 * 64 * 2 / (res["v_fma_f32"]["ms"] * 1e-3) / 1e12, 1)
    # what the rotation alone costs on the value workload: one slice per 16 elements
    r = res["rht128_slice"]
    r["us_for_8192x8192"] = round(r["ms"] * 1e3 * (8192 * 8192 / 16 / 64) / (waves * iters), 2)
    ms = t_ms(lambda i: qii.qii_microbench(qii.MB_MFMA_F16, None, b, 0, blocks, iters))
    res["v_mfma_f32_32x32x16_f16"] = {"ms": round(ms, 4), "TFLOPs": round(waves * iters * 4 * 2 * 32 * 32 * 16 / (ms * 1e-3) / 1e12, 1)}
    # the GEMM's inner loop without its memory side: one block per compute unit, one wave per SIMD
    res["gemm_inner_loop_no_memory"] = {}
    for chunks, cname in ((0, "matrix_instructions_only"), (1, "with_dequantization_as_in_the_gemm"),
                          (2, "with_one_operand_dequantized"), (3, "with_dequantization_from_packed_e2m3"),
                          (4, "matrix_instructions_only_changing_operands")):
        ms = t_ms(lambda i: qii.qii_microbench(qii.MB_MFMA_DEQUANT, None, b, chunks, 256, 4096))
        res["gemm_inner_loop_no_memory"][cname] = {"ms": round(ms, 4), "TFLOPs": round(256 * 4 * 4096 * 16 * 2 * 32 * 32 * 16 / (ms * 1e-3) / 1e12, 1)}
    # launch floor and atomics: the extra time per block over an empty kernel of the same grid
    res["atomics"] = {}
    for blocks in (4096, 16384, 65536):
        e = t_ms(lambda i: qii.qii_microbench(qii.MB_EMPTY, None, None, 0, blocks, 0))
        one = t_ms(lambda i: qii.qii_microbench(qii.MB_ATOMIC_ONE_WORD, b, None, 0, blocks, 0))
        spread = t_ms(lambda i: qii.qii_microbench(qii.MB_ATOMIC_SPREAD, b, None, 0, blocks, 0))
        res["atomics"][f"blocks_{blocks}"] = {"empty_kernel_us": round(e * 1e3, 2), "one_word_us": round(one * 1e3, 2),
                                              "spread_64_words_us": round(spread * 1e3, 2),
                                              "ns_per_atomic_one_word": round((one - e) * 1e6 / blocks, 2),
                                              "ns_per_atomic_spread": round((spread - e) * 1e6 / blocks, 2)}
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three device copies of 512 MiB (untimed) so that a profiler's "
                         "HBM byte counters can be scaled against a transfer of known size")
    ap.add_argument("--quant-rows", type=int, default=8192)
    ap.add_argument("--quant-cols", type=int, default=8192)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--d-in", type=int, default=2048)
    ap.add_argument("--d-out", type=int, default=8192)
    ap.add_argument("--parts", choices=["all", "roofline", "quantize", "linear"], default="all",
                    help="run only the two abs-max-supplied launches behind `roofline` and `roofline_cols`, only the quantize-only parts or only the layer parts of a step (for profiles in "
                         "which every launch of a kernel has the same tensor size); the JSON line then reports "
                         "the skipped parts as null timings")
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="skip what runs after the timed steps: the larger configurations (the decoder's linears at "
                         "32768 tokens, the two stress shapes) and the paper's table of Llama-like layer shapes (App. D) "
                         "at 8 x 2048 tokens next to plain bf16 matmuls of the same shapes (torch.matmul, i.e. the vendor "
                         "GEMM library, the 'speedup over BF16' denominator)")
    ap.add_argument("--microbench", action="store_true",
                    help="instead of the benchmark, measure the machine limits the rooflines are argued from (streaming "
                         "rates, the quantizer's traffic pattern without arithmetic, instruction issue rates, atomics) "
                         "and print them as one JSON line")
    ap.add_argument("--paper-shapes", action="store_true", help="(kept for compatibility: the table is part of the default run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2601_22813_amd import binding as qii
    from paper_2601_22813_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qii.lib()  # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.microbench:
        print(json.dumps({"microbench": microbench(torch, qii, dev)}))
        return 0

    def to_dev(bits: np.ndarray) -> torch.Tensor:
        return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)

    # ------------------------------------------------------------------ part A buffers
    R, C = args.quant_rows, args.quant_cols
    x_np = synth.student_t_bf16((R, C), 3, 0.1, seed=1)
    n_rot = max(2, int(np.ceil(768 * 2 ** 20 / (R * C * 2))))
    xs = [to_dev(x_np)]
    for i in range(1, n_rot):
        xs.append(torch.roll(xs[0], shifts=17 * i, dims=0).contiguous())
    out_rows = qii.NVFP4Tensor.empty(R, C)
    out_cols = qii.NVFP4Tensor.empty(C, R)
    amax = torch.zeros(1, dtype=torch.float32, device=dev)
    # abs-max of every rotating buffer in both layouts, measured once, outside the timed region
    amax_rows = [torch.zeros(1, dtype=torch.float32, device=dev) for _ in xs]
    amax_cols = [torch.zeros(1, dtype=torch.float32, device=dev) for _ in xs]
    for x, ar, ac in zip(xs, amax_rows, amax_cols):
        qii.qii_absmax(x, False, 128, 0, ar)
        qii.qii_absmax(x, True, 128, 0, ac)

    # ------------------------------------------------------------------ part B buffers
    T, d_in, d_out = args.tokens, args.d_in, args.d_out
    X_np, W_np, E_np = synth.linear_layer_bf16(T, d_in, d_out, seed=2)
    Xs, Ws, Es = [to_dev(X_np)], [to_dev(W_np)], [to_dev(E_np)]
    for i in range(1, 3):
        Xs.append(torch.roll(Xs[0], 5 * i, 0).contiguous())
        Ws.append(torch.roll(Ws[0], 5 * i, 0).contiguous())
        Es.append(torch.roll(Es[0], 5 * i, 0).contiguous())
    Xq, Wq = qii.NVFP4Tensor.empty(T, d_in), qii.NVFP4Tensor.empty(d_out, d_in)
    Y = torch.empty((T, d_out), dtype=torch.bfloat16, device=dev)
    dX = torch.empty((T, d_in), dtype=torch.bfloat16, device=dev)
    dW = torch.empty((d_out, d_in), dtype=torch.bfloat16, device=dev)
    ws_f = torch.empty(qii.qii_linear_fwd_workspace_bytes(T, d_in, d_out), dtype=torch.uint8, device=dev)
    amax_X = [torch.zeros(1, dtype=torch.float32, device=dev) for _ in Xs]
    amax_W = [torch.zeros(1, dtype=torch.float32, device=dev) for _ in Ws]
    for x_, w_, ax_, aw_ in zip(Xs, Ws, amax_X, amax_W):   # measured once, outside the timed region
        qii.qii_absmax(x_, False, 0, 0, ax_)
        qii.qii_absmax(w_, False, 0, 0, aw_)
    ws_b = torch.empty(qii.qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, qii.MS_EDEN_PH), dtype=torch.uint8, device=dev)
    ws_ph = torch.empty(qii.qii_quantize_posthoc_workspace_bytes(max(R, C), max(R, C)), dtype=torch.uint8, device=dev)
    ws_pair = torch.empty(qii.qii_quantize_pair_workspace_bytes(R, C, qii.MS_EDEN_PH), dtype=torch.uint8, device=dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    names = ["single_rows", "single_cols", "absmax_rows", "quant_rows", "absmax_cols", "quant_cols",
             "posthoc_rows", "posthoc_cols", "pair_ph", "pair_alg1", "linear_fwd", "linear_bwd", "linear_fwd_46",
             "linear_bwd_ph", "linear_fwd_46_amax"]
    kernel_ms = {k: [] for k in names}

    do_v = args.parts in ("all", "roofline", "quantize")     # the two single-pass launches behind `roofline` / `roofline_cols`
    do_q, do_l = args.parts in ("all", "quantize"), args.parts in ("all", "linear")

    kBatch = 4

    def step(i: int, record: bool):
        e = [ev() for _ in range(len(names) + 1)]
        a, b, c, d = (i * 4) % n_rot, (i * 4 + 1) % n_rot, (i * 4 + 2) % n_rot, (i * 4 + 3) % n_rot
        # A1: kBatch launches of each kernel back to back on kBatch different cold buffers, one event pair around
        # the batch: the per-launch figure then carries the gap between consecutive kernels on the GPU (about 1 us)
        # instead of the host's event and launch overhead (several us), and agrees with the profiler's kernel duration
        e[0].record()
        if do_v:
            for k in range(kBatch):
                j = (i * 4 + k) % n_rot
                qii.qii_quantize_nvfp4(xs[j], False, qii.MS_EDEN, 128, 0, i, amax_rows[j], out_rows, None)
        e[1].record()
        if do_v:
            for k in range(kBatch):
                j = (i * 4 + 2 + k) % n_rot
                qii.qii_quantize_nvfp4(xs[j], True, qii.MS_EDEN, 128, 0, i, amax_cols[j], out_cols, None)
        e[2].record()
        if do_q:
            qii.qii_absmax(xs[c], False, 128, 0, amax)
        e[3].record()
        if do_q:
            qii.qii_quantize_nvfp4(xs[c], False, qii.MS_EDEN, 128, 0, i, amax, out_rows, None)
        e[4].record()
        if do_q:
            qii.qii_absmax(xs[d], True, 128, 0, amax)
        e[5].record()
        if do_q:
            qii.qii_quantize_nvfp4(xs[d], True, qii.MS_EDEN, 128, 0, i, amax, out_cols, None)
        e[6].record()
        # the same two tensors without a known abs-max, in the two-kernel form of Sec. 7
        if do_q:
            qii.qii_quantize_nvfp4(xs[a], False, qii.MS_EDEN_PH, 128, 0, i, None, out_rows, ws_ph)
        e[7].record()
        if do_q:
            qii.qii_quantize_nvfp4(xs[b], True, qii.MS_EDEN_PH, 128, 0, i, None, out_cols, ws_ph)
        e[8].record()
        # both orientations of one tensor from a single read (the backward pass's Q(E), Q(E^T)): the
        # post hoc form (one heavy pass + two scales passes) and Algorithm 1 (two abs-max passes + one read)
        if do_q:
            qii.qii_quantize_pair_nvfp4(xs[c], qii.MS_EDEN_PH, 0, i, 1, i + 1, out_rows, out_cols, ws_pair)
        e[9].record()
        if do_q:
            qii.qii_quantize_pair_nvfp4(xs[d], qii.MS_EDEN, 0, i, 1, i + 1, out_rows, out_cols, ws_pair)
        e[10].record()
        j = i % 3
        if do_l:
            qii.qii_linear_fwd(Xs[j], Ws[j], Y, Xq, Wq, ws_f)
        e[11].record()
        if do_l:
            qii.qii_linear_bwd(Es[j], Xq, Wq, i, dX, dW, ws_b)
        e[12].record()
        # the layer as the paper runs it: 4/6 on the forward pass, post hoc range alignment on the backward pass
        k = (i + 1) % 3
        if do_l:
            qii.qii_linear_fwd_mode(Xs[k], Ws[k], qii.RTN_46, Y, Xq, Wq, ws_f)
        e[13].record()
        if do_l:
            qii.qii_linear_bwd_mode(Es[k], Xq, Wq, i, qii.MS_EDEN_PH, dX, dW, ws_b)
        e[14].record()
        # the same forward pass when the caller brings max|X| and max|W| (App. D assumes so)
        if do_l:
            qii.qii_linear_fwd_mode(Xs[k], Ws[k], qii.RTN_46, Y, Xq, Wq, ws_f, amax_x=amax_X[k], amax_w=amax_W[k])
        e[15].record()
        return e if record else None

    if args.copy_calibration:
        src = torch.empty(512 * 2 ** 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events = [step(args.warmup + i, True) for i in range(args.steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for e in events:
        for k, name in enumerate(names):
            kernel_ms[name].append(e[k].elapsed_time(e[k + 1]))
    avg = {k: float(np.mean(v)) for k, v in kernel_ms.items()}
    avg["single_rows"] /= kBatch      # per launch
    avg["single_cols"] /= kBatch
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # after the timed steps: the forward GEMM alone (the layer's dominant kernel), for its roofline line
    gemm_ws = torch.empty(max(256, qii.qii_gemm_workspace_bytes(T, d_out, d_in)), dtype=torch.uint8, device=dev)
    gemm_ms = []
    for i in range(6 if do_l else 0):
        e0, e1 = ev(), ev()
        e0.record()
        qii.qii_gemm_nvfp4(Xq, Wq, Y, gemm_ws)
        e1.record()
        torch.cuda.synchronize()
        if i:
            gemm_ms.append(e0.elapsed_time(e1))
    gemm_tflops = 2.0 * T * d_in * d_out / (float(np.mean(gemm_ms)) * 1e-3) / 1e12 if do_l else 0.0

    n = R * C
    bytes_a1 = 2 * n * BYTES_PER_ELEM_QUANT
    value_supplied = bytes_a1 / ((avg["single_rows"] + avg["single_cols"]) * 1e-3) / 1e9
    bytes_a2 = 2 * n * (BYTES_PER_ELEM_ABSMAX + BYTES_PER_ELEM_QUANT)
    ms_a2 = avg["absmax_rows"] + avg["quant_rows"] + avg["absmax_cols"] + avg["quant_cols"]
    quant_kernel_gbps = n * BYTES_PER_ELEM_QUANT / (avg["single_rows"] * 1e-3) / 1e9
    flops = 3 * 2.0 * T * d_in * d_out
    lin_ms = avg["linear_fwd"] + avg["linear_bwd"]
    tflops = flops / (lin_ms * 1e-3) / 1e12
    lin2_ms = avg["linear_fwd_46"] + avg["linear_bwd_ph"]
    tflops2 = flops / (lin2_ms * 1e-3) / 1e12
    lin3_ms = avg["linear_fwd_46_amax"] + avg["linear_bwd_ph"]
    tflops3 = flops / (lin3_ms * 1e-3) / 1e12
    bytes_ph = 2 * n * BYTES_PER_ELEM_POSTHOC
    ms_ph = avg["posthoc_rows"] + avg["posthoc_cols"]
    value = bytes_ph / (ms_ph * 1e-3) / 1e9 if do_q else value_supplied
    quant_cols_gbps = n * BYTES_PER_ELEM_QUANT / (avg["single_cols"] * 1e-3) / 1e9

    result = {
        "metric": "MS-EDEN quantize HBM GB/s; NVFP4 linear fwd+bwd TFLOP/s (% of MFMA peak)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"MS-EDEN quantize of {R}x{C} bf16 0.1*Student-t(3), RHT-128, blocks along "
                        f"rows then columns, cold inputs, no abs-max supplied, in the two-kernel form of Sec. 7 "
                        f"(heavy pass + scales pass; all launches counted) (value); the same with the abs-max "
                        f"supplied (quantize.single_pass_*) and as abs-max pass + quantize pass (quantize.two_pass); "
                        f"plus linear fwd+bwd T={T} d_in={d_in} d_out={d_out} bf16 (linear_fwd_bwd)",
            "quantize_bytes_per_element": {"absmax_pass": BYTES_PER_ELEM_ABSMAX, "quantize_pass": BYTES_PER_ELEM_QUANT,
                                           "post_hoc_both_passes": BYTES_PER_ELEM_POSTHOC},
            "rotating_input_buffers": n_rot,
        },
        "quantize": {
            # abs-max supplied by the caller (App. D): one launch per tensor, 2.5625 B per element
            "abs_max_supplied_GBps": round(value_supplied, 1),
            "single_pass_rows_ms": round(avg["single_rows"], 4), "single_pass_cols_ms": round(avg["single_cols"], 4),
            "single_pass_rows_GBps": round(quant_kernel_gbps, 1),
            "single_pass_cols_GBps": round(n * BYTES_PER_ELEM_QUANT / (avg["single_cols"] * 1e-3) / 1e9, 1),
            "two_pass": {"absmax_rows_ms": round(avg["absmax_rows"], 4), "quantize_rows_ms": round(avg["quant_rows"], 4),
                         "absmax_cols_ms": round(avg["absmax_cols"], 4), "quantize_cols_ms": round(avg["quant_cols"], 4),
                         "GBps": round(bytes_a2 / (ms_a2 * 1e-3) / 1e9, 1)},
            # Sec. 7: heavy pass + scales-only pass instead of abs-max pass + quantize pass
            "post_hoc": {"rows_ms": round(avg["posthoc_rows"], 4), "cols_ms": round(avg["posthoc_cols"], 4),
                         "bytes_per_element": BYTES_PER_ELEM_POSTHOC,
                         "GBps": round(bytes_ph / (ms_ph * 1e-3) / 1e9, 1),
                         "speedup_over_two_pass": round(ms_a2 / ms_ph, 3)},
            # Q(x) and Q(x^T) from one read of x (qii_quantize_pair_nvfp4), against the two separate calls above
            "both_orientations_one_read": {
                "post_hoc_ms": round(avg["pair_ph"], 4), "speedup_over_separate_post_hoc": round(ms_ph / avg["pair_ph"], 3),
                "algorithm1_ms": round(avg["pair_alg1"], 4), "speedup_over_separate_two_pass": round(ms_a2 / avg["pair_alg1"], 3)},
        },
        "linear_fwd_bwd": {
            "value": round(tflops, 1), "unit": "TFLOP/s", "ms": round(lin_ms, 4),
            "fwd_ms": round(avg["linear_fwd"], 4), "bwd_ms": round(avg["linear_bwd"], 4),
            "flop": flops, "mfma": "v_mfma_f32_32x32x16_f16", "peak_TFLOPs": MFMA_F16_PEAK_TFLOPS,
            "frac_of_peak": round(tflops / MFMA_F16_PEAK_TFLOPS, 4),
            "paper_context": "up to 4.2x over BF16 on Blackwell (abstract); another machine, not a target",
            # the layer as the paper runs it: 4/6 forward (Sec. 4.1), post hoc range alignment backward (Sec. 7)
            "with_4over6_fwd_and_post_hoc_bwd": {
                "value": round(tflops2, 1), "unit": "TFLOP/s", "ms": round(lin2_ms, 4),
                "fwd_ms": round(avg["linear_fwd_46"], 4), "bwd_ms": round(avg["linear_bwd_ph"], 4),
                "frac_of_peak": round(tflops2 / MFMA_F16_PEAK_TFLOPS, 4),
                # with max|X| and max|W| supplied by the caller, as the paper's own layer timings assume
                "fwd_ms_absmax_supplied": round(avg["linear_fwd_46_amax"], 4),
                "value_absmax_supplied": round(tflops3, 1),
                "frac_of_peak_absmax_supplied": round(tflops3 / MFMA_F16_PEAK_TFLOPS, 4)},
        },
        "roofline": {
            "kernel": "quantize_rows_kernel<bf16, MS_EDEN, RHT> (abs-max supplied, cold input)",
            "bound": "hbm",
            "achieved": round(quant_kernel_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(quant_kernel_gbps / HBM_PEAK_GBPS, 4),
            # HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by what the same
            # counters read for a 512 MiB device copy (x2.0 and x1.0)
            "traffic": {"bytes": TRAFFIC_QUANT_ROWS_BYTES, "algorithmic_bytes": int(n * BYTES_PER_ELEM_QUANT),
                        "valid_for": "8192x8192 bf16", "source": "profiles/quantize_8192x8192_hbm_traffic.txt"} if (R, C) == (8192, 8192) else None,
        },
        # the same for the columns kernel (transposed source), the slower of the two
        "roofline_cols": {
            "kernel": "quantize_cols_kernel<bf16, MS_EDEN, RHT> (abs-max supplied, cold input)", "bound": "hbm",
            "achieved": round(quant_cols_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(quant_cols_gbps / HBM_PEAK_GBPS, 4),
        },
        # the same launch against the vector-ALU peak: what the arithmetic contract asks per element
        # (7 butterfly add/sub, scaling fma 2, abs/max 1, quotient 1, FP4 rounding 1, two EDEN fma 4,
        # per-group divisions and roundings ~0.5) over the fp32 vector peak (256 CUs x 4 SIMDs x 32
        # lanes x 2 flops of a fused multiply-add x 2.4 GHz = 157.3 TFLOP/s)
        "roofline_alu": {
            "kernel": "quantize_rows_kernel<bf16, MS_EDEN, RHT>", "bound": "alu",
            "achieved": round(n * ALU_FLOPS_PER_ELEM / (avg["single_rows"] * 1e-3) / 1e12, 2),
            "peak": VALU_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(n * ALU_FLOPS_PER_ELEM / (avg["single_rows"] * 1e-3) / 1e12 / VALU_F32_PEAK_TFLOPS, 4),
            "flops_per_element": ALU_FLOPS_PER_ELEM,
            "note": "mostly single adds in binary32 (1 flop per lane-instruction against the 2 of an fma; several "
                    "conversion and cross-lane instructions issue at half or quarter rate); "
                    "the kernel runs within 10 % of its own loads and stores without arithmetic (profiles/microbench_summary.txt)",
        },
        "roofline_gemm": {
            "kernel": f"gemm_kernel_v4<bf16 out> M={T} N={d_out} K={d_in} (incl. the scale re-tiling launch)",
            "bound": "mfma", "achieved": round(gemm_tflops, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(gemm_tflops / MFMA_F16_PEAK_TFLOPS, 4),
        },
    }

    if args.parts != "all":   # partial runs are for profiles: no figures for what did not run
        result["config"]["parts"] = args.parts
        if not do_q:
            result["value"] = None
        if not do_v:
            result["roofline"] = None
            result["roofline_cols"] = None
            result["roofline_alu"] = None
        if not do_q:
            result["quantize"] = None
        if not do_l:
            result["linear_fwd_bwd"] = None
            result["roofline_gemm"] = None
    if not args.no_extra_configs and args.parts == "all":
        # free the step buffers first: the stress shapes need several GiB
        del xs, Xs, Ws, Es, Y, dX, dW, ws_b, ws_ph, ws_pair, out_rows, out_cols
        torch.cuda.empty_cache()
        result["configs"] = large_configs(torch, qii, dev)
        result["paper_shapes"] = paper_shapes(torch, qii, synth, dev)
        result["inexact_gemm"] = inexact_gemm(torch, qii, synth, dev, T, d_in, d_out)

    if not args.no_cpu_baseline and do_q:
        import oracle
        oracle.build()
        reps = 0
        t0 = time.perf_counter()
        while reps < 3 or time.perf_counter() - t0 < 12.0:   # a bounded sample: 12 s or more of oracle time
            for transpose in (False, True):
                oracle.quantize(x_np, oracle.MS_EDEN_PH, transpose=transpose, seed_rht=0, seed_sr=reps)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        result["cpu_baseline"] = {
            "value": round(bytes_ph / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.max_threads(),
            "kind": "oracle",
            "sample": f"the whole `value` workload ({R}x{C} MS-EDEN with post hoc range alignment, rows then "
                      f"columns, same byte count as the GPU figure) {reps} times, {dt:.2f} s of wall time each",
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
