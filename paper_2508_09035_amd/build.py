"""Compile the HIP sources into libpdd.so (gfx950 only), in-tree."""
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libpdd.so")
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libpdd_probe.so")   # measurement helper used by the benchmark

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code only: no NaN bookkeeping (a max of MFMA results otherwise costs an extra
    # canonicalising instruction per operand); NaN inputs are documented as undefined
    "-Xarch_device", "-fno-honor-nans",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _hipcc(out: str, src: str, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", out, os.path.join(CSRC, src)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        lines = [l for l in (res.stdout + res.stderr).splitlines()
                 if "not a recognized feature" not in l]
        print("\n".join(lines))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}")


def build_library(verbose: bool = False) -> str:
    """libpdd.so (the C ABI of include/pdd.h) and libpdd_probe.so (the matrix-pipe probe the
    benchmark reports beside the published peak)."""
    _hipcc(LIB_PATH, "pdd_api.hip", verbose)
    _hipcc(PROBE_LIB_PATH, "mfma_probe.hip", verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
