"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the host code, no GPU:
the C oracle on small inputs through every code path, and the library's host
layer (argument validation, chunk plan, workspace rules) through every kind of
rejected call.  The device code is compiled as usual (sanitizers apply to the
host side only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_04342_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", OMP_NUM_THREADS="4",
               UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)


def test_oracle_under_asan_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-std=c99",
           os.path.join(ROOT, "oracle", "rehyat_oracle.c"),
           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = _run(exe)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitize ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_host_layer_under_asan_ubsan(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "host_san")
    host = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        host += ["-Xarch_host", f]
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host, "-fno-honor-nans",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument"]
    cmd += [os.path.join(CSRC, s) for s in ("rehyat_api.hip", "rehyat_state.hip",
                                            "rehyat_prefix.hip", "rehyat_attn.hip",
                                            "rehyat_grad.hip")]
    cmd += [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=900)
    r = _run(exe)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitize ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
