"""Builds the HIP library (csrc/*.hip -> librsa_hip.so) for gfx950 with hipcc."""
import glob
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "librsa_hip.so")


def sources():
    return sorted(glob.glob(os.path.join(_PKG, "csrc", "*.hip")))


def build(verbose=False):
    """Compile every HIP source for gfx950 into one shared library (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [
        hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-I" + os.path.join(_ROOT, "include"), "-I" + os.path.join(_PKG, "csrc"),
        # packed fp32 VALU forms are switched off on the test machines
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument",
    ] + sources() + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
