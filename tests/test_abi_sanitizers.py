"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU:
a copy of the library with instrumented host code is built, and a plain C program
(tests/abi_sanitize_driver.c) calls every entry point with arguments the validation must reject,
extreme sizes included.  A stray read, an overflow in a size computation or a wrong return code
fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="ROCm clang not found")
def test_argument_checks_under_address_and_ub_sanitizers(tmp_path):
    from paper_2501_12956_amd import build
    out = str(tmp_path / "san")
    lib = build.build_sanitized(out)
    exe = os.path.join(out, "abi_sanitize_driver")
    res = subprocess.run([CLANG, "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                          "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                          os.path.join(ROOT, "tests", "abi_sanitize_driver.c"), "-o", exe,
                          "-L", out, "-lganq_san", "-Wl,-rpath," + out, "-Wl,-rpath,/opt/rocm/lib"],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    env = dict(os.environ)
    # leak checking needs ptrace, which containers often forbid, and is not what is tested here
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    text = run.stdout + run.stderr
    assert run.returncode == 0, text
    assert "AddressSanitizer" not in text and "runtime error" not in text, text
    assert "all calls returned as documented" in run.stdout
    shutil.rmtree(out, ignore_errors=True)
