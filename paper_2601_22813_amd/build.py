"""Build libqii.so (the HIP library behind include/qii.h) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqii.so")
SOURCES = ["api.hip", "quantize.hip", "quantize_rows.hip", "quantize_cols.hip", "quantize_pair.hip", "gemm.hip", "gemm_inexact.hip", "selftest.hip", "microbench.hip"]
HEADERS = ["qii_device.h", "qii_internal.h", "quantize_core.h", "quantize_lanes.h", "gemm_common.h", "gemm_sharing_map.h", os.path.join("..", "..", "include", "qii.h")]

# -ffp-contract=off: the quantizers take integer decisions from binary32 arithmetic whose
# every rounding is part of the contract with the parity oracle; fused operations appear
# only where the source writes them.  Packed-FP32 instruction selection is disabled.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip()]
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and lines:
            print("\n".join(lines))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


def build_sanitized(out_dir: str) -> str:
    """A second build of the library whose HOST half is compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer (the device code is unchanged and never runs in that check), written
    to out_dir/libqii_san.so.  For tests/sanitize/abi_check.c; the product never loads it."""
    os.makedirs(out_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(out_dir, src.replace(".hip", ".san.o"))
        cmd = ["hipcc", *FLAGS, *san, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized host) failed on {src}:\n{out}")
    lib = os.path.join(out_dir, "libqii_san.so")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-gpu-sanitize", "-shared-libsan", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
