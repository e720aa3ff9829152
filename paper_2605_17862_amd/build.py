"""Builds csrc/ into lib/libfopd.so with hipcc for gfx950 (cross-compiles without a GPU)."""

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "lib", "libfopd.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose=False):
    os.makedirs(os.path.dirname(LIB), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
        "-o", LIB, os.path.join(PKG, "csrc", "fopd_api.hip"),
    ]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + err + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libfopd.so")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
