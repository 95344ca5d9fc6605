"""Compile the HIP sources into libpdd.so (gfx950 only), in-tree."""
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libpdd.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, os.path.join(CSRC, "pdd_api.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        lines = [l for l in (res.stdout + res.stderr).splitlines()
                 if "not a recognized feature" not in l]
        print("\n".join(lines))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
