"""Host sanitizer pass (CPU only): the C part of the CPU checker and the host half of the C ABI
(argument validation, scalar helpers) built with AddressSanitizer + UndefinedBehaviorSanitizer
and driven through paths that need no GPU.  A sanitizer report ends the driver with a non-zero
status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def test_oracle_c_under_asan_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "pdd_oracle.c")]
    base = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off"]
    plain, san = str(tmp_path / "plain"), str(tmp_path / "san")
    assert _run(base + src + ["-o", plain, "-lm"]).returncode == 0
    r = _run(base + SAN + src + ["-o", san, "-lm"])
    if r.returncode != 0 and "asan" in r.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert r.returncode == 0, r.stderr
    a = _run([plain])
    b = _run([san], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert a.returncode == 0 and b.returncode == 0, b.stderr[-2000:]
    assert a.stdout == b.stdout and "ragged rc=0" in a.stdout
    assert "runtime error" not in b.stderr and "AddressSanitizer" not in b.stderr


def test_abi_validation_layer_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_san")
    cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp"),
           os.path.join(ROOT, "paper_2508_09035_amd", "csrc", "pdd_api.hip"), "-o", exe]
    r = _run(cmd)
    assert r.returncode == 0, r.stderr[-3000:]
    r = _run([exe])
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
