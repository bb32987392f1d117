"""Host sanitizer jobs (CPU only): the C oracle and the host side of the HIP library are built with
-fsanitize=address,undefined and driven by tests/sanitize/*.  GPU code is not instrumented (the
device pass is compiled as usual); nothing here launches a kernel."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, env=ENV, **kw)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    return out


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-I" + os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "rsa_oracle.c"),
         os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"])
    assert "SANITIZE_ORACLE_OK" in run([exe])


def test_host_logic_of_the_hip_library_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    csrc = os.path.join(ROOT, "paper_2105_13120_amd", "csrc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"] + san
    lib = str(tmp_path / "librsa_hip_san.so")
    srcs = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith(".hip"))
    run(common + ["-fPIC", "-shared"] + srcs + ["-o", lib])
    exe = str(tmp_path / "host_san")
    run(common + ["-x", "hip", os.path.join(SAN, "host_driver.cpp"), "-x", "none", lib, "-Wl,-rpath," + str(tmp_path), "-o", exe])
    assert "SANITIZE_HOST_OK" in run([exe])
