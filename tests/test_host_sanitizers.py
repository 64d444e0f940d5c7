"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; GPU sanitizers are not used):
the C oracle, and the argument-handling layer of the C ABI linked against stub launchers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = os.path.join(ROOT, "tests", "host")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_selftest")
    build = run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-o", exe,
                 os.path.join(HOST, "oracle_selftest.c"), os.path.join(ROOT, "oracle", "hyena_oracle.c"), "-lm"])
    assert build.returncode == 0, build.stderr
    res = run([exe], env=ENV)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "0 problem(s)" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_abi_host_logic_under_asan_ubsan(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "abi_selftest")
    csrc = os.path.join(ROOT, "paper_2503_01868_amd", "csrc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + csrc] + san + [
               os.path.join(csrc, "api.hip"), os.path.join(HOST, "launch_stubs.cpp"), os.path.join(HOST, "abi_selftest.cpp"),
               "-o", exe]
    build = run(cmd)
    assert build.returncode == 0, build.stderr[-3000:]
    res = run([exe], env=ENV)
    # hyena_stream_copy and the "empty dh" path reach the HIP runtime; without a GPU they report a launch error,
    # which the self test treats as a problem only on a machine that has a device
    out = res.stdout + res.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-3000:]
    assert "abi selftest:" in res.stdout, out[-3000:]
