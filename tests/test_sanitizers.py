"""CPU-only sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer, findings abort):
the oracle's C file driven over small exactly sized buffers and edge cases, and the library's
host code (argument validation, workspace and split planning) driven through every refusal
path of the C ABI.  The library is compiled with the sanitizers on its host side only; no
call in the driver reaches the GPU runtime, so the test needs no GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, "%s\n%s" % (" ".join(cmd), p.stdout[-4000:])
    return p.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off",
          "-fsanitize=address,undefined,float-cast-overflow,float-divide-by-zero",
          "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-Werror",
          os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "lbt_oracle.c"),
          "-o", exe, "-lm"])
    out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="4"))
    assert "oracle under sanitizers: ok" in out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_abi_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2407_12637_amd import build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    lib = str(tmp_path / "liblbt_hostsan.so")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-O3", "-Wall")]
    # -O1: the device side is compiled too (the host objects reference its image) but never runs
    _run([HIPCC] + flags + ["-O1", "-w"] + san + ["-o", lib] + build.sources())
    exe = str(tmp_path / "abi_refusals")
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-w"] + san +
         ["-I", os.path.join(ROOT, "include"), "-x", "hip", os.path.join(SAN, "abi_refusals.cpp"),
          "-o", exe, "-L", str(tmp_path), "-llbt_hostsan", "-Wl,-rpath," + str(tmp_path)])
    out = _run([exe], env=ENV)
    assert "abi refusals under sanitizers: ok" in out
    shutil.rmtree(tmp_path, ignore_errors=True)
