"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code: the oracle (C) and the
host half of the HIP library (argument checks, workspace arithmetic).  Each check is a small C
driver under tests/sanitize/ that is built here with the sanitizers, run as its own process, and
must exit cleanly with no report.  No GPU is involved: the library's driver only makes calls that
return before anything is enqueued."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_check")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           os.path.join(ROOT, "tests", "sanitize", "oracle_check.c"), os.path.join(ROOT, "oracle", "qii_oracle.c"),
           "-lm", "-o", exe]
    b = run(cmd)
    assert b.returncode == 0, b.stdout
    r = run([exe], env=dict(ENV, OMP_NUM_THREADS="4"), timeout=300)
    assert r.returncode == 0 and "oracle sanitize: ok" in r.stdout, r.stdout
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to build the library's host code")
def test_library_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2601_22813_amd import build
    lib = build.build_sanitized(str(tmp_path))
    exe = str(tmp_path / "abi_check")
    clang = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    cmd = [clang, "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-shared-libsan",
           os.path.join(ROOT, "tests", "sanitize", "abi_check.c"), lib, f"-Wl,-rpath,{tmp_path}", "-o", exe]
    b = run(cmd)
    assert b.returncode == 0, b.stdout
    rt = run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"]).stdout.strip()
    env = dict(ENV)
    if os.path.sep in rt:
        env["LD_LIBRARY_PATH"] = os.path.dirname(rt) + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    r = run([exe], env=env, timeout=300)
    assert r.returncode == 0 and "abi sanitize: ok" in r.stdout, r.stdout
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, r.stdout
