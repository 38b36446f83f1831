"""The host code of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

Argument validation, workspace planning and the block-rate dynamic programme are plain CPU code; this builds them
with -fsanitize=address,undefined (host side only, the device code is untouched) and runs the two host test files
against that library in a child process that preloads the sanitizer runtime.  No GPU is involved."""
import os
import subprocess
import sys

import pytest

from paper_2509_24899_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sanitized_lib():
    return B.build_sanitized_host_library()


def test_library_is_instrumented(sanitized_lib):
    syms = subprocess.run(["nm", "-D", "--undefined-only", sanitized_lib], check=True, capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms


def test_host_tests_pass_under_asan_and_ubsan(sanitized_lib):
    runtime = B.asan_runtime()
    assert os.path.exists(runtime), runtime
    env = dict(os.environ)
    env["HYBRID_ATTN_LIB"] = sanitized_lib
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # python itself is not instrumented and never frees everything at exit: leak checking would only report it
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_abi_host.py"), os.path.join(ROOT, "tests", "test_rate_select_lib.py")]
    run = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    text = run.stdout + run.stderr
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert run.returncode == 0, text[-4000:]
    assert " passed" in run.stdout
