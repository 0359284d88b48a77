"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the C oracle, the native scheduling simulator
and the host side of the C ABI (workspace sizing and every argument check, which all return before the first HIP call).
Each driver under tests/sanitize/ holds its data in exactly sized heap buffers and exits non-zero on the first report.
GPU code is not instrumented (device sanitizers are not available here); its safety nets are the guard-region and
repeatability tests that run on the GPU."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)      # the sanitizer runtime has to come first in the library list


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "driver_oracle")
    _run(["gcc", *FLAGS, "-static-libasan", "-fopenmp", "-std=c11", "-Wall", os.path.join(SAN, "driver_oracle.c"),
          os.path.join(ROOT, "oracle", "moe_oracle.c"), "-o", exe, "-lm"])
    assert "clean" in _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=1"))


def test_scheduling_simulator_under_sanitizers(tmp_path):
    exe = str(tmp_path / "driver_sched")
    obj = str(tmp_path / "driver_sched.o")
    _run(["gcc", *FLAGS, "-std=c11", "-Wall", "-I", os.path.join(ROOT, "include"), "-c", os.path.join(SAN, "driver_sched.c"), "-o", obj])
    _run(["g++", *FLAGS, "-static-libasan", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"),
          os.path.join(ROOT, "paper_2511_11373_amd", "csrc_host", "mars_sched.cpp"), obj, "-o", exe])
    assert "clean" in _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=1"))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_abi_host_side_under_sanitizers(tmp_path):
    """The library's host code instrumented (-Xarch_host), the device code compiled as usual; the driver only reaches paths that
    return before any HIP call."""
    lib = str(tmp_path / "libmoe_ffn_san.so")
    exe = str(tmp_path / "driver_abi")
    san = [a for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all") for a in ("-Xarch_host", f)]
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2511_11373_amd", "csrc", "*.hip")))
    _run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument", *san, "-I", os.path.join(ROOT, "include"),
          "-I", os.path.join(ROOT, "paper_2511_11373_amd", "csrc"), *srcs, "-o", lib])
    clang = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    _run([clang, *FLAGS, "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "driver_abi.c"), lib, "-Wl,-rpath," + str(tmp_path), "-o", exe])
    assert "clean" in _run([exe], env=ENV)
