"""Builds csrc/ into lib/libfopd.so with hipcc for gfx950 (cross-compiles without a GPU)."""

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "lib", "libfopd.so")
PROBE = os.path.join(PKG, "lib", "hbm_probe")
GEMM_PROBE = os.path.join(PKG, "lib", "gemm_probe")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, what, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"   # the host pass does not know the flag
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + err + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building " + what)


def build_library(verbose=False):
    """Compiles the C-ABI library and the two probe programs.  Returns the library's path."""
    os.makedirs(os.path.dirname(LIB), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + HIPCC_FLAGS + [
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
        "-o", LIB, os.path.join(PKG, "csrc", "fopd_api.hip"),
    ], "libfopd.so", verbose)
    probe_flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    _run([hipcc] + probe_flags + ["-o", PROBE, os.path.join(PKG, "csrc", "hbm_probe.hip")],
         "hbm_probe", verbose)
    _run([hipcc] + probe_flags + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
                                  "-o", GEMM_PROBE, os.path.join(PKG, "csrc", "gemm_probe.hip")],
         "gemm_probe", verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
