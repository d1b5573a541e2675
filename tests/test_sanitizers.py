"""Host-side AddressSanitizer / UndefinedBehaviorSanitizer builds (no GPU): the CPU oracle, and the
argument validation of the C ABI (the library's host code compiled with the sanitizers; the device
code is compiled as usual and never runs here)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
# the environment is passed on as it is; the sanitizer runtime is told not to insist on being loaded first
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fno-fast-math",
         "-ffp-contract=off", "-o", exe, os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "imunpack_oracle.c"),
         "-lm"])
    out = run([exe], env=ENV)
    assert "0 failures" in out and "ERROR" not in out and "runtime error" not in out, out


def test_library_argument_validation_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2403_07339_amd", "csrc")
    lib = str(tmp_path / "libimunpack_san.so")
    srcs = [os.path.join(csrc, f) for f in ("api.hip", "percentile.hip", "quantize.hip", "plan.hip", "unpack.hip", "gemm.hip")]
    run([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
         "-o", lib, *srcs])
    exe = str(tmp_path / "abi_san")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    cc = clang if os.path.exists(clang) else shutil.which("clang") or hipcc
    run([cc, "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"),
         "-o", exe, os.path.join(SAN, "abi_driver.c"), lib, "-Wl,-rpath," + str(tmp_path), "-lm"])
    out = run([exe], env=ENV)
    assert "0 failures" in out and "ERROR: AddressSanitizer" not in out and "runtime error" not in out, out
