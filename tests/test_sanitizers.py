"""CPU builds of the oracle and of the C ABI's host side under AddressSanitizer and
UndefinedBehaviorSanitizer (signed-integer overflow included: all arithmetic is 64-bit integer),
each run over its driver in tests/sanitize/.  No GPU, no GPU code."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fsanitize=signed-integer-overflow",
       "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)


def run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, f"{' '.join(cmd)}\n{p.stdout[-4000:]}"
    return p.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    run(["gcc", "-O1", "-fopenmp", "-Wall", *SAN, "-o", exe,
         os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "ckpt_oracle.c")])
    out = run([exe], env=ENV)
    assert "oracle_driver ok" in out


def test_host_side_of_the_abi_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_driver")
    flags = []
    for f in SAN:
        flags += ["-Xarch_host", f] if f.startswith("-fsanitize") or f.startswith("-fno-sanitize") else [f]
    run([hipcc, "--cuda-host-only", "-x", "hip", "-O1", "-std=c++17", *flags, "-o", exe,
         os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
         os.path.join(ROOT, "paper_2502_12499_amd", "csrc", "ckpt_api.hip"),
         os.path.join(ROOT, "paper_2502_12499_amd", "csrc", "ragged_host.hip")])
    out = run([exe], env=ENV)
    assert "host_driver ok" in out
